"""MI355X-native SART hot path: paged decode attention over reasoning branches
and the prune / finish bookkeeping, as a C-ABI HIP library (libsart.so) with a
thin ctypes binding.  The library must be built (python -m
paper_2505_13326_amd.build or __graft_entry__.build()); there is no fallback."""
from .binding import (  # noqa: F401
    ACTIVE, BF16, COMPLETED, DEFAULT_SKEW_PERMILLE, DROP_LOWEST_K, EARLY_STOPPED, E_HIP, E_INVALID, E_OOM_PAGES, E_STATE, F32,
    FP8_E4M3, KEEP_TOP_K, LAYOUT_MFMA16, LAYOUT_MFMA16_FP8, LAYOUT_NATURAL, OK, PRUNED, SEQ_BRANCH, SEQ_PREFIX, THRESHOLD, UNUSED, WAITING,
    SartCache, SartError, exported_symbols, lib_path, load_library, mfma_probe, read_probe,
)
