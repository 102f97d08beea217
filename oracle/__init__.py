"""ctypes binding of the float64 CPU oracle (sart_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
cpu_baseline leg import this package.  It shares nothing with the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "sart_oracle.c")
_LIB = os.path.join(_DIR, "libsart_oracle.so")

OK, E_INVALID, E_OOM_PAGES, E_STATE = 0, 1, 2, 3
UNUSED, ACTIVE, COMPLETED, PRUNED, EARLY_STOPPED, WAITING = range(6)
SEQ_PREFIX, SEQ_BRANCH = 0, 1
DROP_LOWEST_K, KEEP_TOP_K, THRESHOLD = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        ip, vp, dp, fp = C.POINTER(C.c_int), C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_float)
        L.orc_create.restype = vp
        L.orc_create.argtypes = [C.c_int] * 11 + [ip]
        L.orc_destroy.argtypes = [vp]
        L.orc_append.argtypes = [vp, C.c_int, C.c_int, ip, ip, vp, vp]
        L.orc_attention.argtypes = [vp, vp, C.c_int, C.c_double, ip, C.c_int, dp, dp]
        L.orc_prefill_attention.argtypes = [vp, C.c_int, vp, C.c_int, C.c_double, dp, dp]
        L.orc_finish.argtypes = [vp, C.c_int, ip]
        L.orc_start.argtypes = [vp, C.c_int, ip]
        L.orc_fork.argtypes = [vp, C.c_int, ip, ip]
        L.orc_set_start_waiting.argtypes = [vp, C.c_int]
        L.orc_set_fp8.argtypes = [vp, C.c_double, C.c_double]
        L.orc_fp8_roundtrip.argtypes = [vp, C.c_int, C.c_double, vp, vp]
        L.orc_fp8_roundtrip.restype = None
        L.orc_prune.argtypes = [vp, C.c_int, C.c_int, ip, fp, ip, fp, C.c_int]
        L.orc_request_done.argtypes = [vp, C.c_int]
        L.orc_get_state.argtypes = [vp] + [ip] * 11
        L.orc_get_state.restype = None
        L.orc_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _iptr(a):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int))


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def fp8_roundtrip(bits, scale=1.0):
    """The oracle's E4M3 codec on bf16 bit patterns: (codes uint8, read-back values float64).
    scale is taken as the float32 value a cache description carries."""
    scale = float(np.float32(scale))
    b = np.ascontiguousarray(bits, np.uint16)
    codes = np.zeros(b.size, np.uint8)
    vals = np.zeros(b.size, np.float64)
    _load().orc_fp8_roundtrip(b.ctypes.data, b.size, float(scale), codes.ctypes.data, vals.ctypes.data)
    return codes.reshape(b.shape), vals.reshape(b.shape)


def num_threads() -> int:
    return int(_load().orc_num_threads())


class OracleCache:
    """Plain CPU paged cache + attention.  dtype: 'f32' (float32 arrays),
    'bf16' (uint16 bit arrays) or 'fp8' (uint16 bf16 bit arrays in, the cache
    keeps 8-bit floats)."""

    def __init__(self, *, n_q_heads, n_kv_heads, head_dim, page_tokens, num_pages, max_requests,
                 branches_per_request, finish_quota, max_pages_per_branch, max_prefix_pages, dtype,
                 free_order=None, k_scale=1.0, v_scale=1.0, start_waiting=False):
        self.L = _load()
        self.Hq, self.Hkv, self.d, self.pt = n_q_heads, n_kv_heads, head_dim, page_tokens
        self.num_pages, self.max_req, self.Nb = num_pages, max_requests, branches_per_request
        self.Q, self.max_bp, self.max_pp = finish_quota, max_pages_per_branch, max_prefix_pages
        self.dtype = dtype
        self.np_dtype = np.float32 if dtype == "f32" else np.uint16
        fo = _i32(free_order)
        self.h = self.L.orc_create(n_q_heads, n_kv_heads, head_dim, page_tokens, num_pages, max_requests,
                                   branches_per_request, finish_quota, max_pages_per_branch,
                                   max_prefix_pages, 0 if dtype == "f32" else 1, _iptr(fo))
        if not self.h:
            raise ValueError("orc_create rejected the description")
        if start_waiting:       # a request's branches are created WAITING and join the batch through start()
            assert self.L.orc_set_start_waiting(self.h, 1) == OK
        if dtype == "fp8":      # bf16 in and out, K and V kept as 8-bit floats (E4M3) of x / scale
            # a cache description carries its scales as float32
            if self.L.orc_set_fp8(self.h, float(np.float32(k_scale)), float(np.float32(v_scale))) != OK:
                raise ValueError("orc_set_fp8 rejected the scales")

    def close(self):
        if self.h:
            self.L.orc_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _raw(self, x, shape_tail):
        x = np.ascontiguousarray(x, dtype=self.np_dtype)
        assert x.shape[1:] == tuple(shape_tail), (x.shape, shape_tail)
        return x

    def append(self, kind, ids, n_tokens, k, v) -> int:
        ids_a, nt_a = _i32(ids), _i32(n_tokens)
        k = self._raw(k, (self.Hkv, self.d))
        v = self._raw(v, (self.Hkv, self.d))
        n_seqs = len(ids_a) if ids_a is not None else (len(nt_a) if nt_a is not None else k.shape[0])
        total = int(nt_a.sum()) if nt_a is not None else n_seqs
        assert k.shape[0] == total and v.shape[0] == total, (k.shape, total)
        return self.L.orc_append(self.h, kind, n_seqs, _iptr(ids_a), _iptr(nt_a),
                                 k.ctypes.data, v.ctypes.data)

    def attention(self, q, scale=0.0, rows=None, want_wsum=False):
        q = self._raw(q, (self.Hq, self.d))
        rows_a = _i32(rows)
        n_out = len(rows_a) if rows_a is not None else self.n_active
        out = np.zeros((n_out, self.Hq, self.d), dtype=np.float64)
        ws = np.zeros((n_out, self.Hq), dtype=np.float64)
        rc = self.L.orc_attention(self.h, q.ctypes.data, q.shape[0], float(scale), _iptr(rows_a), n_out,
                                  out.ctypes.data_as(C.POINTER(C.c_double)),
                                  ws.ctypes.data_as(C.POINTER(C.c_double)))
        if rc != OK:
            raise ValueError(f"orc_attention status {rc}")
        return (out, ws) if want_wsum else out

    def prefill_attention(self, request, q, scale=0.0, want_wsum=False):
        """Causal attention of the last len(q) prompt tokens of `request` (Algorithm 1, Prefill).
        Returns a status code on error, else out [n_q, Hq, d] float64 (and the weight sums)."""
        q = self._raw(q, (self.Hq, self.d))
        n_q = q.shape[0]
        out = np.zeros((n_q, self.Hq, self.d), dtype=np.float64)
        ws = np.zeros((n_q, self.Hq), dtype=np.float64)
        rc = self.L.orc_prefill_attention(self.h, int(request), q.ctypes.data, n_q, float(scale),
                                          out.ctypes.data_as(C.POINTER(C.c_double)),
                                          ws.ctypes.data_as(C.POINTER(C.c_double)))
        if rc != OK:
            return rc
        return (out, ws) if want_wsum else out

    def start(self, handles) -> int:
        """Waiting branches join the batch (Algorithm 1, main workflow)."""
        h = _i32(handles)
        return self.L.orc_start(self.h, len(h), _iptr(h))

    def fork(self, src, dst) -> int:
        """Branches split: dst[i] (WAITING) joins the batch as a copy of src[i] (ACTIVE), sharing its full pages."""
        s_, d_ = _i32(src), _i32(dst)
        if len(s_) != len(d_):
            return E_INVALID
        return self.L.orc_fork(self.h, len(s_), _iptr(s_), _iptr(d_))

    def finish(self, handles) -> int:
        h = _i32(handles)
        return self.L.orc_finish(self.h, len(h), _iptr(h))

    def prune(self, mode, scores, k=0, k_per_request=None, threshold=None, max_pruned=None) -> int:
        s = np.ascontiguousarray(scores, dtype=np.float32)
        kp, mp = _i32(k_per_request), _i32(max_pruned)
        th = None if threshold is None else np.ascontiguousarray(threshold, dtype=np.float32)
        fp = C.POINTER(C.c_float)
        return self.L.orc_prune(self.h, mode, int(k), _iptr(kp),
                                None if th is None else th.ctypes.data_as(fp), _iptr(mp),
                                s.ctypes.data_as(fp), len(s))

    def request_done(self, r) -> bool:
        return bool(self.L.orc_request_done(self.h, int(r)))

    @property
    def n_active(self) -> int:
        n = C.c_int(0)
        self.L.orc_get_state(self.h, C.byref(n), *([None] * 10))
        return n.value

    def state(self) -> dict:
        H = self.max_req * self.Nb
        st = {
            "n_active": np.zeros(1, np.int32),
            "active_handles": np.zeros(H, np.int32),
            "seq_lens": np.zeros(H, np.int32),
            "block_tables": np.zeros((H, self.max_bp), np.int32),
            "free_stack": np.zeros(self.num_pages, np.int32),
            "free_top": np.zeros(1, np.int32),
            "prefix_tables": np.zeros((self.max_req, self.max_pp), np.int32),
            "prefix_lens": np.zeros(self.max_req, np.int32),
            "prefix_refcnt": np.zeros(self.max_req, np.int32),
            "branch_state": np.zeros(H, np.int32),
            "req_counters": np.zeros((self.max_req, 2), np.int32),
        }
        self.L.orc_get_state(self.h, *[_iptr(st[k]) for k in (
            "n_active", "active_handles", "seq_lens", "block_tables", "free_stack", "free_top",
            "prefix_tables", "prefix_lens", "prefix_refcnt", "branch_state", "req_counters")])
        return st
