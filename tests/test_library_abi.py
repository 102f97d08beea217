"""The C-ABI library loads without a GPU and exports every symbol the headers
under include/ declare; host-side argument checks that need no device."""
import ctypes as C
import os
import re

import paper_2505_13326_amd as sart

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(sart_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert "sart_alloc_cache" in names and "sart_decode_attention" in names and len(names) >= 12
    lib = C.CDLL(sart.lib_path())
    for n in names:
        assert hasattr(lib, n), n
    assert names == sart.exported_symbols()


def test_pool_bytes_and_null_checks_need_no_gpu():
    lib = sart.load_library()
    from paper_2505_13326_amd.binding import _Desc
    d = _Desc(1, 28, 4, 128, 16, 1000, 16, 8, 0, 1025, 32, sart.BF16, 0, None, 0, None, 1.0, 1.0, 0)
    assert lib.sart_pool_bytes(C.byref(d)) == 1000 * 16 * 2 * 4 * 128 * 2
    out = C.c_void_p()
    d.n_q_heads = 30  # not a multiple of the KV heads
    assert lib.sart_alloc_cache(C.byref(d), C.byref(out)) == sart.E_INVALID
    assert b"multiple" in lib.sart_last_error()
    assert lib.sart_append_tokens(None, 0, 0, None, None, None, None, 0, None) == sart.E_INVALID
    assert lib.sart_sync_status(None) == sart.E_INVALID
