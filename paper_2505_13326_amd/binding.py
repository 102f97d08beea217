"""ctypes binding of libsart.so: argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams,
nothing else); every step of the path runs in the library's HIP kernels.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

OK, E_INVALID, E_OOM_PAGES, E_STATE, E_HIP = range(5)
F32, BF16, FP8_E4M3 = 0, 1, 2
SEQ_PREFIX, SEQ_BRANCH = 0, 1
UNUSED, ACTIVE, COMPLETED, PRUNED, EARLY_STOPPED, WAITING = range(6)
DROP_LOWEST_K, KEEP_TOP_K, THRESHOLD = 0, 1, 2
LAYOUT_NATURAL, LAYOUT_MFMA16, LAYOUT_MFMA16_FP8 = 0, 1, 2
DEFAULT_SKEW_PERMILLE = 80   # the library's default of sart_set_decode_launch's skew_permille

_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_DIR, "libsart.so")
_lib = None

_ip = C.POINTER(C.c_int32)
_fp = C.POINTER(C.c_float)


class SartError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"sart status {status}: {message}")
        self.status = status


class _Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_tokens", C.c_int32), ("num_pages", C.c_int32),
                ("max_requests", C.c_int32), ("branches_per_request", C.c_int32),
                ("finish_quota", C.c_int32), ("max_pages_per_branch", C.c_int32),
                ("max_prefix_pages", C.c_int32), ("kv_dtype", C.c_int32),
                ("force_natural_layout", C.c_int32), ("kv_pool", C.c_void_p),
                ("kv_pool_bytes", C.c_size_t), ("initial_free_order", _ip), ("k_scale", C.c_float),
                ("v_scale", C.c_float), ("branches_start_waiting", C.c_int32)]


class _Policy(C.Structure):
    _fields_ = [("mode", C.c_int32), ("k", C.c_int32), ("k_per_request", _ip), ("threshold", _fp),
                ("max_pruned", _ip)]


_SIGNATURES = {
    "sart_pool_bytes": (C.c_size_t, [C.POINTER(_Desc)]),
    "sart_alloc_cache": (C.c_int, [C.POINTER(_Desc), C.POINTER(C.c_void_p)]),
    "sart_free_cache": (C.c_int, [C.c_void_p]),
    "sart_cache_layout": (C.c_int32, [C.c_void_p]),
    "sart_append_tokens": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, _ip, _ip, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_void_p]),
    "sart_decode_attention": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_float,
                                        C.c_void_p]),
    "sart_decode_attention_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_float,
                                               C.c_void_p]),
    "sart_prefill_attention": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, _ip, _ip, C.c_void_p, C.c_void_p, C.c_float,
                                         C.c_void_p]),
    "sart_prune_branches": (C.c_int, [C.c_void_p, C.POINTER(_Policy), C.c_void_p, C.c_int32, C.c_void_p]),
    "sart_finish_branch": (C.c_int, [C.c_void_p, C.c_int32, _ip, C.c_void_p]),
    "sart_start_branches": (C.c_int, [C.c_void_p, C.c_int32, _ip, C.c_void_p]),
    "sart_fork_branches": (C.c_int, [C.c_void_p, C.c_int32, _ip, _ip, C.c_void_p]),
    "sart_finish_reached": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "sart_append_active_by_handle": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "sart_decode_attention_by_handle": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]),
    "sart_active_count_hint": (C.c_int32, [C.c_void_p]),
    "sart_device_views": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]),
    "sart_sync_status": (C.c_int, [C.c_void_p]),
    "sart_get_state": (C.c_int, [C.c_void_p] + [_ip] * 11),
    "sart_set_profiling": (C.c_int, [C.c_void_p, C.c_int32]),
    "sart_last_decode_ms": (C.c_int, [C.c_void_p, _fp, _fp]),
    "sart_set_decode_launch": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]),
    "sart_set_merge_mode": (C.c_int, [C.c_void_p, C.c_int32]),
    "sart_set_prompt_stagger": (C.c_int, [C.c_void_p, C.c_int32]),
    "sart_read_probe": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "sart_mfma_probe": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "sart_read_probe_shaped": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_void_p]),
    "sart_last_error": (C.c_char_p, []),
}


def exported_symbols():
    """Names the header declares; the loader resolves every one of them."""
    return sorted(_SIGNATURES)


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libsart.so.  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_13326_amd.build`")
        lib = C.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)  # AttributeError if the symbol is not exported
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def read_probe(buf, chunk_order=None, stream=None, shape=None):
    """sart_read_probe over a torch device tensor (measurement aid).  shape: (workgroups, depth, flavour,
    interleave) of sart_read_probe_shaped, or None for the default probe."""
    lib = load_library()
    order = None if chunk_order is None else C.c_void_p(chunk_order.data_ptr())
    if shape is None:
        rc = lib.sart_read_probe(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), order, _stream_handle(stream))
    else:
        rc = lib.sart_read_probe_shaped(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), order,
                                        *[int(x) for x in shape], _stream_handle(stream))
    if rc != OK:
        raise SartError(rc, lib.sart_last_error().decode())


def mfma_probe(operands, rounds, n_workgroups, sink, shape=0, stream=None):
    """sart_mfma_probe over torch device tensors (measurement aid): operands 16 KiB, sink n_workgroups * 256 floats."""
    lib = load_library()
    assert operands.numel() * operands.element_size() >= 16384 and sink.numel() >= n_workgroups * 256 and sink.element_size() == 4
    rc = lib.sart_mfma_probe(C.c_void_p(operands.data_ptr()), int(rounds), int(n_workgroups), int(shape), C.c_void_p(sink.data_ptr()),
                             _stream_handle(stream))
    if rc != OK:
        raise SartError(rc, lib.sart_last_error().decode())


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a, typ=_ip):
    return None if a is None else a.ctypes.data_as(typ)


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class SartCache:
    """One paged KV cache with its branch tables (wraps sart_cache*)."""

    def __init__(self, *, n_q_heads, n_kv_heads, head_dim, page_tokens=16, num_pages, max_requests,
                 branches_per_request, finish_quota=0, max_pages_per_branch, max_prefix_pages, dtype="bf16",
                 free_order=None, kv_pool=None, force_natural_layout=False, n_layers=1, k_scale=1.0, v_scale=1.0,
                 start_waiting=False):
        import torch
        self.lib = load_library()
        self.Hq, self.Hkv, self.d, self.pt = n_q_heads, n_kv_heads, head_dim, page_tokens
        self.num_pages, self.max_req, self.Nb = num_pages, max_requests, branches_per_request
        self.Q, self.max_bp, self.max_pp = finish_quota, max_pages_per_branch, max_prefix_pages
        self.dtype = dtype
        self.torch_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        self.n_layers = n_layers
        d = _Desc(n_layers, n_q_heads, n_kv_heads, head_dim, page_tokens, num_pages, max_requests, branches_per_request,
                  finish_quota, max_pages_per_branch, max_prefix_pages, {"f32": F32, "bf16": BF16, "fp8": FP8_E4M3}[dtype],
                  1 if force_natural_layout else 0, None, 0, None, float(k_scale), float(v_scale), 1 if start_waiting else 0)
        self.pool_bytes = int(self.lib.sart_pool_bytes(C.byref(d)))
        self._pool = kv_pool  # keep the tensor alive
        if kv_pool is not None:
            d.kv_pool = C.c_void_p(kv_pool.data_ptr())
            d.kv_pool_bytes = kv_pool.numel() * kv_pool.element_size()
        fo = _i32(free_order)
        if fo is not None:
            d.initial_free_order = _ptr(fo)
        h = C.c_void_p()
        self._check(self.lib.sart_alloc_cache(C.byref(d), C.byref(h)))
        self.h = h
        self.layout = int(self.lib.sart_cache_layout(self.h))

    # -- plumbing -----------------------------------------------------------
    def _check(self, rc):
        if rc != OK:
            raise SartError(rc, self.lib.sart_last_error().decode())

    def close(self):
        if getattr(self, "h", None):
            self.lib.sart_free_cache(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _dev(self, x, tail):
        """numpy (f32 / bf16 bits) or torch tensor -> contiguous device tensor of the cache dtype."""
        import torch
        if isinstance(x, np.ndarray):
            if self.dtype == "f32":
                t = torch.from_numpy(np.ascontiguousarray(x, np.float32))
            else:
                t = torch.from_numpy(np.ascontiguousarray(x, np.uint16).view(np.int16)).view(torch.bfloat16)
            x = t.cuda()
        assert x.is_cuda and x.dtype == self.torch_dtype and tuple(x.shape[1:]) == tuple(tail), (x.shape, x.dtype)
        return x.contiguous()

    # -- the five calls -----------------------------------------------------
    def append_tokens(self, kind, ids, n_tokens, k, v, stream=None, status=False, all_active=False, layer=0):
        """sart_append_tokens.  k, v: [sum n, Hkv, d] device tensors (or numpy, copied to the device).
        all_active: SART_ALL_ACTIVE (one token per active branch, count read on the device; k, v hold
        at least that many rows)."""
        ids_a, nt_a = _i32(ids), _i32(n_tokens)
        k = self._dev(k, (self.Hkv, self.d))
        v = self._dev(v, (self.Hkv, self.d))
        if all_active:
            assert ids is None and n_tokens is None and k.shape == v.shape and k.shape[0] >= 1
            rc = self.lib.sart_append_tokens(self.h, kind, -int(k.shape[0]), None, None, C.c_void_p(k.data_ptr()),
                                             C.c_void_p(v.data_ptr()), int(layer), _stream_handle(stream))
            if status:
                return rc if rc != OK else self.sync_status()
            self._check(rc)
            return OK
        n_seqs = len(ids_a) if ids_a is not None else (len(nt_a) if nt_a is not None else k.shape[0])
        total = int(nt_a.sum()) if nt_a is not None else n_seqs
        if k.shape[0] != total or v.shape[0] != total:
            raise ValueError(f"k/v rows {k.shape[0]} != tokens {total}")
        rc = self.lib.sart_append_tokens(self.h, kind, n_seqs, _ptr(ids_a), _ptr(nt_a), C.c_void_p(k.data_ptr()),
                                         C.c_void_p(v.data_ptr()), int(layer), _stream_handle(stream))
        if status:
            return rc if rc != OK else self.sync_status()
        self._check(rc)
        return OK

    def decode_attention(self, q, out=None, scale=0.0, stream=None, layer=0, static_scratch=False):
        """sart_decode_attention (static_scratch: sart_decode_attention_static, which needs `out` from the
        caller since it allocates nothing).  q: [n_rows, Hq, d]; returns out [n_rows, Hq, d] float32 (device)."""
        import torch
        q = self._dev(q, (self.Hq, self.d))
        if out is None:
            assert not static_scratch
            out = torch.zeros((q.shape[0], self.Hq, self.d), dtype=torch.float32, device=q.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
        fn = self.lib.sart_decode_attention_static if static_scratch else self.lib.sart_decode_attention
        self._check(fn(self.h, int(layer), C.c_void_p(q.data_ptr()), C.c_void_p(out.data_ptr()), q.shape[0], float(scale),
                       _stream_handle(stream)))
        return out

    def prefill_attention(self, request_ids, n_q, q, out=None, scale=0.0, stream=None, status=False, layer=0):
        """sart_prefill_attention.  q: [sum n_q, Hq, d], rows in list order; returns out float32 (device)."""
        import torch
        ids, nq = _i32(request_ids), _i32(n_q)
        assert len(ids) == len(nq)
        q = self._dev(q, (self.Hq, self.d))
        assert q.shape[0] == int(np.maximum(nq, 0).sum())
        if out is None:
            out = torch.zeros((q.shape[0], self.Hq, self.d), dtype=torch.float32, device=q.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
        rc = self.lib.sart_prefill_attention(self.h, int(layer), len(ids), _ptr(ids), _ptr(nq), C.c_void_p(q.data_ptr()),
                                             C.c_void_p(out.data_ptr()), float(scale), _stream_handle(stream))
        if status:
            return rc
        self._check(rc)
        return out

    def prune_branches(self, mode, scores, k=0, k_per_request=None, threshold=None, max_pruned=None, stream=None,
                       status=False):
        import torch
        if isinstance(scores, np.ndarray):
            scores = torch.from_numpy(np.ascontiguousarray(scores, np.float32)).cuda()
        assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous()
        kp, mp = _i32(k_per_request), _i32(max_pruned)
        th = None if threshold is None else np.ascontiguousarray(threshold, np.float32)
        for arr in (kp, mp, th):
            if arr is not None and len(arr) != self.max_req:
                raise ValueError("per-request policy arrays need max_requests entries")
        pol = _Policy(int(mode), int(k), _ptr(kp), _ptr(th, _fp), _ptr(mp))
        rc = self.lib.sart_prune_branches(self.h, C.byref(pol), C.c_void_p(scores.data_ptr()), scores.numel(),
                                          _stream_handle(stream))
        if status:
            return rc if rc != OK else self.sync_status()
        self._check(rc)
        return OK

    def start_branches(self, handles, stream=None, status=False):
        """sart_start_branches: waiting branches join the batch."""
        h = _i32(handles)
        rc = self.lib.sart_start_branches(self.h, len(h), _ptr(h), _stream_handle(stream))
        if status:
            return rc if rc != OK else self.sync_status()
        self._check(rc)
        return OK

    def fork_branches(self, src, dst, stream=None, status=False):
        """sart_fork_branches: dst[i] (waiting) joins the batch as a copy of src[i] (active), sharing its full pages."""
        s_, d_ = _i32(src), _i32(dst)
        if len(s_) != len(d_):
            raise ValueError("src and dst differ in length")
        rc = self.lib.sart_fork_branches(self.h, len(s_), _ptr(s_), _ptr(d_), _stream_handle(stream))
        if status:
            return rc if rc != OK else self.sync_status()
        self._check(rc)
        return OK

    def finish_branch(self, handles, stream=None, status=False):
        h = _i32(handles)
        rc = self.lib.sart_finish_branch(self.h, len(h), _ptr(h), _stream_handle(stream))
        if status:
            return rc if rc != OK else self.sync_status()
        self._check(rc)
        return OK

    # -- readback -------------------------------------------------------------
    def finish_reached(self, target_len, stream=None):
        """sart_finish_reached.  target_len: int32 device tensor [max_requests * Nb] by handle."""
        import torch
        assert target_len.is_cuda and target_len.dtype == torch.int32 and target_len.is_contiguous()
        assert target_len.numel() == self.max_req * self.Nb
        self._check(self.lib.sart_finish_reached(self.h, C.c_void_p(target_len.data_ptr()), _stream_handle(stream)))

    def append_active_by_handle(self, k, v, stream=None, layer=0):
        """sart_append_active_by_handle.  k, v: device tensors [max_requests * Nb, Hkv, d], row = branch handle."""
        k = self._dev(k, (self.Hkv, self.d))
        v = self._dev(v, (self.Hkv, self.d))
        assert k.shape[0] == v.shape[0] == self.max_req * self.Nb
        self._check(self.lib.sart_append_active_by_handle(self.h, C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr()), int(layer),
                                                          _stream_handle(stream)))

    def decode_attention_by_handle(self, q, out, scale=0.0, stream=None, layer=0):
        """sart_decode_attention_by_handle.  q, out: device tensors [max_requests * Nb, Hq, d], row = branch handle;
        rows of branches that are not active are left as they are."""
        import torch
        q = self._dev(q, (self.Hq, self.d))
        assert q.shape[0] == self.max_req * self.Nb
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
        self._check(self.lib.sart_decode_attention_by_handle(self.h, int(layer), C.c_void_p(q.data_ptr()),
                                                             C.c_void_p(out.data_ptr()), float(scale), _stream_handle(stream)))
        return out

    def active_count_hint(self) -> int:
        """sart_active_count_hint: the active count without waiting for the device (it lags queued calls)."""
        return int(self.lib.sart_active_count_hint(self.h))

    def device_views(self):
        """sart_device_views as torch int32 tensors over the library's memory (read-only by convention):
        (active handles [max_requests * Nb], active count [1])."""
        import torch
        a, n = C.c_void_p(), C.c_void_p()
        self._check(self.lib.sart_device_views(self.h, C.byref(a), C.byref(n)))

        class _View:
            def __init__(self, ptr, count):
                self.__cuda_array_interface__ = {"shape": (count,), "typestr": "<i4", "data": (ptr, False), "version": 2}
        H = self.max_req * self.Nb
        return (torch.as_tensor(_View(a.value, H), device="cuda"), torch.as_tensor(_View(n.value, 1), device="cuda"))

    def sync_status(self) -> int:
        return int(self.lib.sart_sync_status(self.h))

    _STATE_FIELDS = ("n_active", "active_handles", "seq_lens", "block_tables", "free_stack", "free_top",
                     "prefix_tables", "prefix_lens", "prefix_refcnt", "branch_state", "req_counters")

    def get_state(self, with_status=False, fields=None):
        """sart_get_state (synchronises).  fields: names to read back (default: all); a step loop that only
        needs the active list should not copy the block tables."""
        H = self.max_req * self.Nb
        shapes = {
            "n_active": 1, "active_handles": H, "seq_lens": H, "block_tables": (H, self.max_bp),
            "free_stack": self.num_pages, "free_top": 1, "prefix_tables": (self.max_req, self.max_pp),
            "prefix_lens": self.max_req, "prefix_refcnt": self.max_req, "branch_state": H,
            "req_counters": (self.max_req, 2),
        }
        want = self._STATE_FIELDS if fields is None else tuple(fields)
        assert all(f in shapes for f in want)
        st = {k: np.zeros(shapes[k], np.int32) for k in want}
        rc = self.lib.sart_get_state(self.h, *[_ptr(st[k]) if k in st else None for k in self._STATE_FIELDS])
        if rc == E_HIP:
            self._check(rc)
        return (st, int(rc)) if with_status else st

    @property
    def n_active(self) -> int:
        n = C.c_int32(0)
        self.lib.sart_get_state(self.h, C.byref(n), *([None] * 10))
        return n.value

    # -- measurement / tuning -------------------------------------------------
    def set_profiling(self, repeats: int):
        self._check(self.lib.sart_set_profiling(self.h, int(repeats)))

    def set_prompt_stagger(self, on: bool):
        self._check(self.lib.sart_set_prompt_stagger(self.h, 1 if on else 0))

    def set_merge_mode(self, in_kernel: bool):
        self._check(self.lib.sart_set_merge_mode(self.h, 1 if in_kernel else 0))

    def last_decode_ms(self):
        a, t = C.c_float(0), C.c_float(0)
        self._check(self.lib.sart_last_decode_ms(self.h, C.byref(a), C.byref(t)))
        return a.value, t.value

    def set_decode_launch(self, n_workgroups=0, prompt_mode=-1, skew_permille=DEFAULT_SKEW_PERMILLE):
        self._check(self.lib.sart_set_decode_launch(self.h, int(n_workgroups), int(prompt_mode), int(skew_permille)))
