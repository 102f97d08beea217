"""Several layers over one set of tables: a token has the same page and slot in
every layer, the layer-0 append allocates, the other layers' appends write only.
One oracle per layer (each repeats the bookkeeping) is the reference."""
import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import GpuEngine, TOL, dims
from helpers import assert_state_equal

pytestmark = pytest.mark.gpu


def test_three_layers_share_tables_and_keep_their_own_kv():
    NL = 3
    base = wl.scaled(wl.CONFIGS[2], n_requests=3, nb=4, prompt_len=70, length_params=(120, 0.8), length_cap=700)
    cfgs = [wl.scaled(base, cfg_id=base.cfg_id + 100 * l) for l in range(NL)]    # another seed per layer
    L = wl.lengths(base)
    pages = wl.pages_needed(base, L, growth_tokens=8) + 4
    kw = dims(base, pages, int(-(-(L.max() + 8) // 16)) + 1)
    fo = wl.free_order(base, pages)
    os_ = [orc.OracleCache(free_order=fo, **kw) for _ in range(NL)]
    g = GpuEngine(free_order=fo, n_layers=NL, **kw)

    def append(kind, ids, ns, kv_of_layer):
        for l in range(NL):
            k, v = kv_of_layer(l)
            assert os_[l].append(kind, ids, ns, k, v) == orc.OK
            g.c.append_tokens(kind, ids, ns, k, v, layer=l)
        assert g.c.sync_status() == 0

    for r in range(base.n_requests):
        append(orc.SEQ_PREFIX, [r], [base.prompt_len], lambda l: wl.prefix_kv(cfgs[l], r))
        ids = [r * base.nb + j for j in range(base.nb)]
        ns = [int(L[r, j]) for j in range(base.nb)]
        append(orc.SEQ_BRANCH, ids, ns, lambda l: tuple(np.concatenate(x) for x in zip(*[wl.branch_kv(cfgs[l], b, n) for b, n in zip(ids, ns)])))
    for l in range(NL):
        assert_state_equal(os_[l].state(), g.state())

    def check_all_layers(step):
        st = os_[0].state()
        act = st["active_handles"][:int(st["n_active"][0])]
        for l in range(NL):
            q = wl.query(cfgs[l], step)[act]
            ref = os_[l].attention(q)
            got = g.c.decode_attention(q, layer=l).cpu().numpy().astype(np.float64)
            err = float(np.abs(got - ref).max())
            assert err <= TOL["bf16"], f"layer {l}: max abs err {err}"
        # prefill attention reads its layer too
        for l in (0, NL - 1):
            q = wl.prefix_query(cfgs[l], 1)
            got = g.c.prefill_attention([1], [base.prompt_len], q, layer=l).cpu().numpy().astype(np.float64)
            assert float(np.abs(got - os_[l].prefill_attention(1, q)).max()) <= TOL["bf16"]
        return act

    act = check_all_layers(0)
    # decode steps: explicit list, default list, all-active form
    for step, form in ((1, "ids"), (2, "default"), (3, "all")):
        for l in range(NL):
            k, v = wl.step_kv(cfgs[l], step)
            assert os_[l].append(orc.SEQ_BRANCH, None, None, k[act], v[act]) == orc.OK
            if form == "ids":
                g.c.append_tokens(orc.SEQ_BRANCH, act, None, k[act], v[act], layer=l)
            elif form == "default":
                g.c.append_tokens(orc.SEQ_BRANCH, None, None, k[act], v[act], layer=l)
            else:
                g.c.append_tokens(orc.SEQ_BRANCH, None, None, k[act], v[act], layer=l, all_active=True)
        assert g.c.sync_status() == 0
        assert_state_equal(os_[0].state(), g.state())
        check_all_layers(step)
    # an append to another layer must repeat the layer-0 append ...
    k, v = wl.step_kv(cfgs[1], 4)
    assert g.c.append_tokens(orc.SEQ_BRANCH, act[:3], None, k[act[:3]], v[act[:3]], layer=1, status=True) == orc.E_INVALID
    assert g.c.append_tokens(orc.SEQ_BRANCH, None, None, k[act], v[act], layer=NL, status=True) == orc.E_INVALID
    # ... a different list of the same length is refused at once too ...
    swapped = act.copy()
    swapped[[0, 1]] = swapped[[1, 0]]
    k0, v0 = wl.step_kv(cfgs[0], 4)
    g.c.append_tokens(orc.SEQ_BRANCH, act, None, k0[act], v0[act], layer=0)
    for l in range(NL):
        kk, vv = wl.step_kv(cfgs[l], 4)
        assert os_[l].append(orc.SEQ_BRANCH, None, None, kk[act], vv[act]) == orc.OK
    assert g.c.append_tokens(orc.SEQ_BRANCH, swapped, None, k[swapped], v[swapped], layer=1, status=True) == orc.E_INVALID
    for l in range(1, NL):
        kk, vv = wl.step_kv(cfgs[l], 4)
        g.c.append_tokens(orc.SEQ_BRANCH, act, None, kk[act], vv[act], layer=l)
    assert g.c.sync_status() == 0
    check_all_layers(4)
    # ... and after a call that moved rows nothing is written (layer 1 keeps its data) and the caller is told
    fin = [int(act[0])]
    for l in range(NL):
        assert os_[l].finish(fin) == orc.OK
    assert g.finish(fin) == orc.OK
    g.c.append_tokens(orc.SEQ_BRANCH, act, None, k[act], v[act], layer=1)
    assert g.c.sync_status() == orc.E_STATE
    assert g.c.sync_status() == 0
    assert_state_equal(os_[0].state(), g.state())
    check_all_layers(5)
