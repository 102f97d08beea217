"""Helpers of the GPU parity tests: build the same seeded state in the oracle
and in the HIP library, and compare."""
import numpy as np

import oracle as orc
import workloads as wl

TOL = {"f32": 1e-5, "bf16": 1e-2}   # max-abs error bounds of the benchmark spec


def _sart():
    import paper_2505_13326_amd as sart
    return sart


class GpuEngine:
    """The HIP library behind the interface the golden runner and the fuzz use."""

    def __init__(self, **kw):
        self.c = _sart().SartCache(**kw)

    def append(self, kind, ids, n_tokens, k, v):
        try:
            return self.c.append_tokens(kind, ids, n_tokens, k, v, status=True)
        except ValueError:
            return orc.E_INVALID

    def prune(self, mode, scores, k=0, k_per_request=None, threshold=None, max_pruned=None):
        return self.c.prune_branches(mode, np.asarray(scores, np.float32), k=k, k_per_request=k_per_request,
                                     threshold=threshold, max_pruned=max_pruned, status=True)

    def finish(self, handles):
        return self.c.finish_branch(handles, status=True)

    def start(self, handles):
        try:
            return self.c.start_branches(handles, status=True)
        except Exception as e:                       # host-side refusals (duplicates, range) are statuses here
            return getattr(e, "status", orc.E_INVALID)

    def fork(self, src, dst):
        try:
            return self.c.fork_branches(src, dst, status=True)
        except Exception as e:                       # host-side refusals are statuses here
            return getattr(e, "status", orc.E_INVALID)

    def state(self):
        return self.c.get_state()


def dims(cfg, num_pages, max_bp, max_pp=None, max_req=None):
    pt = cfg.page_tokens
    return dict(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, page_tokens=pt,
                num_pages=num_pages, max_requests=max_req or cfg.n_requests, branches_per_request=cfg.nb,
                finish_quota=cfg.quota, max_pages_per_branch=max_bp,
                max_prefix_pages=max_pp or max(1, -(-cfg.prompt_len // pt)), dtype=cfg.dtype)


def populate(cfg, engines, L=None, requests=None):
    """Appends every request's prompt and every branch's initial tokens to each
    engine in `engines` (objects with .append like OracleCache / GpuEngine)."""
    L = wl.lengths(cfg) if L is None else L
    reqs = range(cfg.n_requests) if requests is None else requests
    for r in reqs:
        k, v = wl.prefix_kv(cfg, r)
        for e in engines:
            assert e.append(orc.SEQ_PREFIX, [r], [cfg.prompt_len], k, v) == orc.OK
        ks, vs, ids, ns = [], [], [], []
        for j in range(cfg.nb):
            b = r * cfg.nb + j
            kb, vb = wl.branch_kv(cfg, b, int(L[r, j]))
            ks.append(kb); vs.append(vb); ids.append(b); ns.append(int(L[r, j]))
        k, v = np.concatenate(ks), np.concatenate(vs)
        for e in engines:
            assert e.append(orc.SEQ_BRANCH, ids, ns, k, v) == orc.OK


def compare_attention(cfg, o, g, q_by_handle, rows=None, tol=None):
    """Runs one decode attention on both sides with the same queries (gathered
    in active order) and returns the max abs error."""
    st = o.state()
    nA = int(st["n_active"][0])
    act = st["active_handles"][:nA]
    q = q_by_handle[act]
    ref = o.attention(q, rows=rows)
    out = g.c.decode_attention(q).cpu().numpy().astype(np.float64)
    assert g.c.sync_status() == 0
    assert np.all(np.isfinite(out))
    got = out if rows is None else out[np.asarray(rows)]
    err = float(np.abs(got - ref).max()) if got.size else 0.0
    tol = TOL[cfg.dtype] if tol is None else tol
    assert err <= tol, f"max abs err {err} > {tol}"
    return err
