"""Seeded synthetic inputs shaped like the paper's serving workloads.

This module holds data recipes only: branch lengths, completion targets,
reward scores and Q/K/V values.  It contains none of the method's arithmetic
(no attention, no paging, no pruning) and is the one module that both the CPU
oracle's tests and the HIP path's tests/benchmarks read.

The paper serves reasoning models whose responses run to thousands of tokens
with a heavy tail (Section 3, Observation 1; Section 5.2 speaks of 7K-8K token
bins), samples N = 8 branches and early-stops after M = 4 (Figure 3 caption),
and scores branches with a reward in [0, 1] (threshold alpha = 0.5,
Section 5.1).  Its datasets and models are not available here, so every value
below is drawn from a counter-addressed PCG64 stream:

    Generator(PCG64(SeedSequence([BASE_SEED + cfg_id, stream_kind, index])))

Each (kind, index) is its own stream, so any branch's data can be regenerated
without drawing the others (full-size parity samples need this).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 2505133260

# stream kinds
_S_LENGTHS, _S_TARGETS, _S_SCORES, _S_PREFIX, _S_BRANCH, _S_QUERY, _S_STEP_KV, _S_PERM, _S_PREFIX_Q = range(9)


def _rng(cfg_id: int, kind: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED + cfg_id, kind, index])))


# --------------------------------------------------------------------------
# bf16 <-> f32 bit conversions (input quantisation; inputs are *defined* as the
# bf16-rounded values, both sides read the same bits)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Config:
    cfg_id: int
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    n_requests: int       # R
    nb: int               # branches sampled per request (paper's N)
    quota: int            # completions that trigger early stop (paper's M); 0 = off
    prompt_len: int       # P
    length_dist: str      # "uniform" | "lognormal" | "pareto"
    length_params: tuple  # see lengths()
    length_cap: int
    page_tokens: int = 16
    # trace-only fields
    n_steps: int = 1
    prune_every: int = 0
    prune_k: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def token_bytes(self) -> int:
        """KV bytes per token (K and V, all KV heads)."""
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    @property
    def n_handles(self) -> int:
        return self.n_requests * self.nb


CONFIGS = {
    1: Config(1, "tiny", 4, 1, 64, "f32", 1, 4, 0, 128, "uniform", (1, 256), 256),
    2: Config(2, "7b-like", 28, 4, 128, "bf16", 16, 8, 0, 512, "lognormal", (4096, 0.8), 16384),
    3: Config(3, "trace-7b", 28, 4, 128, "bf16", 32, 8, 4, 512, "lognormal", (2048, 0.8), 16384,
              n_steps=400, prune_every=50, prune_k=2),
    4: Config(4, "32b-like", 40, 8, 128, "bf16", 64, 4, 0, 1024, "lognormal", (8192, 0.7), 32768),
    5: Config(5, "heavy-tail", 28, 4, 128, "bf16", 1, 64, 0, 2048, "pareto", (1.5, 64), 32768),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of cfg with some fields replaced (smaller parity cases)."""
    d = {f: getattr(cfg, f) for f in cfg.__dataclass_fields__}
    d.update(kw)
    return Config(**d)


# --------------------------------------------------------------------------
# integer / score draws
# --------------------------------------------------------------------------
def lengths(cfg: Config) -> np.ndarray:
    """Private tokens per branch at the start, int64 [R, Nb]."""
    g = _rng(cfg.cfg_id, _S_LENGTHS)
    shape = (cfg.n_requests, cfg.nb)
    if cfg.length_dist == "uniform":
        lo, hi = cfg.length_params
        L = g.integers(lo, hi + 1, size=shape)
    elif cfg.length_dist == "lognormal":
        med, sigma = cfg.length_params
        L = np.rint(med * np.exp(sigma * g.standard_normal(shape)))
    elif cfg.length_dist == "pareto":
        alpha, xmin = cfg.length_params
        u = 1.0 - g.random(shape)  # (0, 1]
        L = np.floor(xmin * u ** (-1.0 / alpha))
    else:
        raise ValueError(cfg.length_dist)
    return np.clip(L, 1, cfg.length_cap).astype(np.int64)


def remaining_tokens(cfg: Config) -> np.ndarray:
    """Trace workloads: tokens each branch still generates before it completes,
    int64 [R, Nb]: max(1, ceil(100 * exp(0.8 z)))."""
    g = _rng(cfg.cfg_id, _S_TARGETS)
    z = g.standard_normal((cfg.n_requests, cfg.nb))
    return np.maximum(1, np.ceil(100.0 * np.exp(0.8 * z))).astype(np.int64)


def scores(cfg: Config, event: int) -> np.ndarray:
    """Reward stand-ins for prune event `event`: float32 U[0,1) by handle."""
    return _rng(cfg.cfg_id, _S_SCORES, event).random(cfg.n_handles, dtype=np.float32)


def free_order(cfg: Config, num_pages: int) -> np.ndarray:
    """A seeded permutation of the pool's pages (a long-running server's pool
    is scattered)."""
    return _rng(cfg.cfg_id, _S_PERM).permutation(num_pages).astype(np.int32)


# --------------------------------------------------------------------------
# tensors.  Storage form: float32 arrays for "f32", uint16 bf16 bits for "bf16"
# --------------------------------------------------------------------------
def _normal(cfg: Config, g: np.random.Generator, shape) -> np.ndarray:
    x = g.standard_normal(shape, dtype=np.float32)
    return x if cfg.dtype == "f32" else f32_to_bf16_bits(x)


def prefix_kv(cfg: Config, request: int, n_tokens: int | None = None):
    """Prompt K, V of a request: two arrays [P, Hkv, d]."""
    n = cfg.prompt_len if n_tokens is None else n_tokens
    g = _rng(cfg.cfg_id, _S_PREFIX, request)
    kv = _normal(cfg, g, (2, n, cfg.n_kv_heads, cfg.head_dim))
    return kv[0], kv[1]


def prefix_query(cfg: Config, request: int, n_tokens: int | None = None) -> np.ndarray:
    """Queries of a request's prompt tokens (prefill): [P, Hq, d]; a prefix of
    the same stream for a shorter prompt."""
    n = cfg.prompt_len if n_tokens is None else n_tokens
    g = _rng(cfg.cfg_id, _S_PREFIX_Q, request)
    return _normal(cfg, g, (n, cfg.n_q_heads, cfg.head_dim))


def branch_kv(cfg: Config, handle: int, n_tokens: int):
    """Initial private K, V of a branch: two arrays [n_tokens, Hkv, d]."""
    g = _rng(cfg.cfg_id, _S_BRANCH, handle)
    kv = _normal(cfg, g, (2, n_tokens, cfg.n_kv_heads, cfg.head_dim))
    return kv[0], kv[1]


def step_kv(cfg: Config, step: int):
    """K, V of the token every branch would append at decode step `step`,
    indexed by handle: two arrays [R*Nb, Hkv, d]."""
    g = _rng(cfg.cfg_id, _S_STEP_KV, step)
    kv = _normal(cfg, g, (2, cfg.n_handles, cfg.n_kv_heads, cfg.head_dim))
    return kv[0], kv[1]


def query(cfg: Config, step: int) -> np.ndarray:
    """Queries of decode step `step`, indexed by handle: [R*Nb, Hq, d]."""
    g = _rng(cfg.cfg_id, _S_QUERY, step)
    return _normal(cfg, g, (cfg.n_handles, cfg.n_q_heads, cfg.head_dim))


def to_float64(cfg: Config, x: np.ndarray) -> np.ndarray:
    """Exact widening of a stored array to float64 (for dense checks)."""
    return (x if cfg.dtype == "f32" else bf16_bits_to_f32(x)).astype(np.float64)


# --------------------------------------------------------------------------
# pool sizing helpers (plain arithmetic on the draws)
# --------------------------------------------------------------------------
def pages_needed(cfg: Config, L: np.ndarray | None = None, growth_tokens: int = 0) -> int:
    """Pages the initial state occupies (+ room for growth_tokens per branch)."""
    L = lengths(cfg) if L is None else L
    pt = cfg.page_tokens
    private = int(np.sum((L + growth_tokens + pt - 1) // pt))
    prefix = cfg.n_requests * ((cfg.prompt_len + pt - 1) // pt)
    return private + prefix


def unique_kv_bytes(cfg: Config, seq_lens, prefix_lens_live) -> int:
    """Algorithmic KV bytes of one decode step: every live prompt once plus
    every active branch's private tokens."""
    return int((int(np.sum(seq_lens)) + int(np.sum(prefix_lens_live))) * cfg.token_bytes)
