"""Decode attention on inputs built to stress the online softmax and the merge of
partial results: running maxima that rise with every page, pieces whose maxima
are tens of binary orders apart, weights that underflow, one dominant key at the
very end of a long branch, equal keys, a context of a single prompt token, and
one very long branch beside many short ones.  Each case runs under the two
ways the matrix-core kernel reads the shared prompt and is compared with the
float64 oracle (and with the closed form where there is one) at the bf16 bound."""
import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import TOL, GpuEngine, dims

pytestmark = pytest.mark.gpu

HQ, HKV, D = 28, 4, 128
G = HQ // HKV
PROMPT_MODES = {"per-branch": 1, "shared-rows": 2}


def _bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, np.float32))


def _f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def _pair(n_req, nb, P, Lmax, pages):
    cfg = wl.scaled(wl.CONFIGS[2], n_q_heads=HQ, n_kv_heads=HKV, head_dim=D, n_requests=n_req, nb=nb, prompt_len=P)
    kw = dims(cfg, pages, -(-Lmax // 16) + 1, max_pp=max(1, -(-P // 16)))
    fo = np.random.default_rng(pages).permutation(pages).astype(np.int32)
    return cfg, orc.OracleCache(free_order=fo, **kw), GpuEngine(free_order=fo, **kw)


def _both(o, g, kind, ids, ns, k, v):
    assert o.append(kind, ids, ns, k, v) == orc.OK
    assert g.append(kind, ids, ns, k, v) == orc.OK


def _check(o, g, q, mode, launches=((0, 80), (64, 0), (7, 300))):
    """Oracle vs GPU for every active row, under the default launch and two that cut the rows elsewhere."""
    ref = o.attention(q)
    worst = 0.0
    for n_wg, skew in launches:
        g.c.set_decode_launch(n_wg, PROMPT_MODES[mode], skew)
        outs = []
        for in_kernel in (False, True):           # merged by the merge kernel / by the attention kernel's last writers
            g.c.set_merge_mode(in_kernel)
            got = g.c.decode_attention(q).cpu().numpy()
            assert g.c.sync_status() == 0 and np.all(np.isfinite(got))
            worst = max(worst, float(np.abs(got.astype(np.float64) - ref).max()))
            outs.append(got)
        assert np.array_equal(outs[0], outs[1])   # same fold order: the same bits
    g.c.set_merge_mode(False)
    assert worst <= TOL["bf16"], f"max abs err {worst}"
    return ref, worst


@pytest.mark.parametrize("mode", list(PROMPT_MODES))
def test_scores_rising_along_the_context(mode):
    """Every key is a multiple of one direction and every query points along it, so the score of token t is
    c * beta_t with beta rising steadily over prompt and private tokens: every page raises the running
    maximum, the early pieces' maxima lie far below the last piece's (their weights underflow to 0 in
    the merge) and only the last tokens carry weight."""
    rng = np.random.default_rng(11)
    P, Ls = 200, [1500, 700, 333]
    cfg, o, g = _pair(2, 3, P, max(Ls), 2 * (P // 16 + 1) + 2 * sum(-(-l // 16) for l in Ls) + 8)
    u = rng.standard_normal(D)
    u /= np.linalg.norm(u)
    for r in range(2):
        T = P + max(Ls)
        beta_all = np.linspace(-40.0, 40.0, T)                      # scores from -40 c' to +40 c' along the context
        kp = _bf16(beta_all[:P, None, None] * u[None, None, :] * np.ones((1, HKV, 1)))
        vp = _bf16(rng.standard_normal((P, HKV, D)))
        _both(o, g, orc.SEQ_PREFIX, [r], [P], kp, vp)
        for j, L in enumerate(Ls):
            kb = _bf16(beta_all[P:P + L, None, None] * u[None, None, :] * np.ones((1, HKV, 1)))
            vb = _bf16(rng.standard_normal((L, HKV, D)))
            _both(o, g, orc.SEQ_BRANCH, [r * 3 + j], [L], kb, vb)
    # |q| = 30 => score = 30 * beta / sqrt(128) = 2.65 beta: about 3.8 binary orders per unit of beta,
    # 300 binary orders between the first and the last token, 0.2 per token
    q = _bf16(np.broadcast_to(30.0 * u, (6, HQ, D)) * (1 + 0.05 * rng.random((6, HQ, 1))))
    ref, err = _check(o, g, q, mode)
    print(f"rising scores [{mode}]: max abs err {err:.3g}")


@pytest.mark.parametrize("mode", list(PROMPT_MODES))
def test_one_dominant_key_in_the_last_page(mode):
    """Random keys, except that the very last token of each branch has a key along the query with a score
    far above all others: the output must be that token's V row (every other piece's weight underflows)."""
    rng = np.random.default_rng(12)
    P, Ls = 96, [4097, 1030, 17]
    cfg, o, g = _pair(1, 3, P, max(Ls), P // 16 + sum(-(-l // 16) for l in Ls) + 8)
    u = rng.standard_normal(D)
    u /= np.linalg.norm(u)
    _both(o, g, orc.SEQ_PREFIX, [0], [P], _bf16(rng.standard_normal((P, HKV, D))), _bf16(rng.standard_normal((P, HKV, D))))
    last_v = []
    for j, L in enumerate(Ls):
        kb = rng.standard_normal((L, HKV, D))
        kb[-1] = 60.0 * u                                           # score 60 * 40 / sqrt(128) = 212 against ~ +-10
        vb = _bf16(rng.standard_normal((L, HKV, D)))
        last_v.append(_f64(vb[-1]))
        _both(o, g, orc.SEQ_BRANCH, [j], [L], _bf16(kb), vb)
    q = _bf16(np.broadcast_to(40.0 * u, (3, HQ, D)))
    ref, err = _check(o, g, q, mode)
    for j in range(3):                                              # closed form: the dominant token's V row
        want = np.repeat(last_v[j], G, axis=0)
        assert np.abs(ref[j] - want).max() < 1e-9
    print(f"dominant last key [{mode}]: max abs err {err:.3g}")


@pytest.mark.parametrize("mode", list(PROMPT_MODES))
def test_equal_keys_give_the_mean_of_v(mode):
    rng = np.random.default_rng(13)
    P, Ls = 50, [900, 16, 1]
    cfg, o, g = _pair(1, 3, P, max(Ls), P // 16 + 1 + sum(-(-l // 16) for l in Ls) + 8)
    key = _bf16(rng.standard_normal((1, HKV, D)))
    vp = _bf16(rng.standard_normal((P, HKV, D)))
    _both(o, g, orc.SEQ_PREFIX, [0], [P], np.repeat(key, P, axis=0), vp)
    means = []
    for j, L in enumerate(Ls):
        vb = _bf16(rng.standard_normal((L, HKV, D)))
        _both(o, g, orc.SEQ_BRANCH, [j], [L], np.repeat(key, L, axis=0), vb)
        means.append(np.concatenate([_f64(vp), _f64(vb)]).mean(axis=0))
    q = _bf16(rng.standard_normal((3, HQ, D)))
    ref, err = _check(o, g, q, mode)
    for j in range(3):
        assert np.abs(ref[j] - np.repeat(means[j], G, axis=0)).max() < 1e-12     # the oracle against the closed form
    print(f"equal keys [{mode}]: max abs err {err:.3g}")


@pytest.mark.parametrize("mode", list(PROMPT_MODES))
def test_contexts_of_one_prompt_token_and_of_nothing(mode):
    """Request 0: a 1-token prompt and branches without private tokens (the output is that token's V);
    request 1: no prompt, one branch with a single private token, one with none (a zero row)."""
    rng = np.random.default_rng(14)
    cfg, o, g = _pair(2, 2, 1, 16, 16)
    k1, v1 = _bf16(rng.standard_normal((1, HKV, D))), _bf16(rng.standard_normal((1, HKV, D)))
    z = np.zeros((0, HKV, D), np.uint16)
    _both(o, g, orc.SEQ_PREFIX, [0], [1], k1, v1)
    _both(o, g, orc.SEQ_PREFIX, [1], [0], z, z)
    kb, vb = _bf16(rng.standard_normal((1, HKV, D))), _bf16(rng.standard_normal((1, HKV, D)))
    _both(o, g, orc.SEQ_BRANCH, [2], [1], kb, vb)
    q = _bf16(rng.standard_normal((4, HQ, D)))
    ref, err = _check(o, g, q, mode, launches=((0, 80), (3, 0)))
    want = np.repeat(_f64(v1[0]), G, axis=0)
    assert np.abs(ref[0] - want).max() == 0 and np.abs(ref[1] - want).max() == 0
    assert np.abs(ref[2] - np.repeat(_f64(vb[0]), G, axis=0)).max() == 0 and np.all(ref[3] == 0)
    got = g.c.decode_attention(q).cpu().numpy()
    assert np.all(got[3] == 0)


@pytest.mark.parametrize("mode", list(PROMPT_MODES))
def test_one_very_long_branch_beside_63_short_ones(mode):
    """The heavy-tail configuration's intent, drawn explicitly: 1 request x 64 branches sharing a 2048-token
    prompt, one branch at the 32768-token cap, the others 64..400 tokens: the long branch is cut over
    hundreds of waves, the short ones share waves."""
    base = wl.CONFIGS[5]
    rng = np.random.default_rng(15)
    L = rng.integers(64, 401, size=(1, base.nb))
    L[0, 37] = base.length_cap
    pages = wl.pages_needed(base, L) + 8
    kw = dims(base, pages, base.length_cap // 16 + 1)
    fo = wl.free_order(base, pages)
    o, g = orc.OracleCache(free_order=fo, **kw), GpuEngine(free_order=fo, **kw)
    pk, pv = wl.prefix_kv(base, 0)
    _both(o, g, orc.SEQ_PREFIX, [0], [base.prompt_len], pk, pv)
    ids = list(range(base.nb))
    kv = [wl.branch_kv(base, b, int(L[0, b])) for b in ids]
    _both(o, g, orc.SEQ_BRANCH, ids, [int(x) for x in L[0]], np.concatenate([x[0] for x in kv]), np.concatenate([x[1] for x in kv]))
    q = wl.query(base, 0)
    ref, err = _check(o, g, q, mode, launches=((0, 80),))
    print(f"one 32768-token branch beside 63 short ones [{mode}]: max abs err {err:.3g}")
