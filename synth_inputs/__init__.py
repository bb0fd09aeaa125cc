"""Seeded synthetic relay caches (K, V, observation-window queries, budgets).

This module only draws random tensors with the shapes and value structure of
the workloads; it holds none of the method's arithmetic.  Both the CPU oracle's
tests and the GPU tests/bench read their inputs from here so that the two sides
see identical bits.

Recipe (per (layer, kv_head), every tensor has its own PCG64 stream seeded by
SeedSequence([seed, base_config, layer, kv_head, tensor_id])):

* "iid"        : fp32 i.i.d. N(0,1) K, V, Q_win; per KV head `heavy` distinct
                 token indices whose key rows are scaled by `heavy_scale`.
* "structured" : X = (sqrt(.5) E + sqrt(.5) (F G)/sqrt(lowrank)) * s, with
                 E [N,d], F [N,lowrank], G [lowrank,d] i.i.d. N(0,1) and
                 s_c = exp(0.5 z_c) a per-channel log-normal scale; K and V are
                 drawn independently.  Optionally a set of round(frac*N)
                 outlier tokens per layer (shared by K, V and all heads of the
                 layer) has its rows scaled by `outlier_scale`.
                 Q_win is i.i.d. N(0,1).
All draws are float32; the result is rounded once (RNE) to the I/O dtype.
bf16 tensors are returned as uint16 bit patterns.
"""
from __future__ import annotations

import concurrent.futures as _cf
from dataclasses import dataclass, replace
from typing import Dict, Iterable, Optional, Tuple

import numpy as np

_T_K, _T_V, _T_Q, _T_HEAVY, _T_BUDGET = 0, 1, 2, 3, 4
_OUTLIER_HEAD = 0xFFFF


@dataclass(frozen=True)
class RelayConfig:
    name: str
    base: int                 # seeding id: shadow configs share their base config's data
    n_layers: int
    n_kv_heads: int
    group: int                # query heads per KV head
    head_dim: int
    n_tokens: int
    window: int
    budget: int               # uniform budget; ignored when budget_range is set
    rank: int
    dtype: str                # "f32" | "bf16"
    dist: str                 # "iid" | "structured"
    heavy: int = 0
    heavy_scale: float = 1.0
    lowrank: int = 16
    outlier_frac: float = 0.0
    outlier_scale: float = 8.0
    budget_range: Optional[Tuple[float, float]] = None   # per-head budgets = round(U[lo,hi]*N)
    budget_int_range: Optional[Tuple[int, int]] = None   # per-head budgets = U{lo..hi}
    agents: int = 1           # sequential independent calls, seeds seed..seed+agents-1

    @property
    def n_heads(self) -> int:
        return self.n_layers * self.n_kv_heads

    @property
    def n_q_heads(self) -> int:
        return self.n_kv_heads * self.group

    @property
    def rows(self) -> int:    # window-query rows per KV head
        return self.group * self.window


def _named() -> Dict[str, RelayConfig]:
    c: Dict[str, RelayConfig] = {}
    c["1"] = RelayConfig("1", 1, 1, 2, 2, 64, 512, 16, 64, 1, "f32", "iid", heavy=8, heavy_scale=4.0)
    c["2"] = RelayConfig("2", 2, 36, 8, 4, 128, 2048, 32, 205, 4, "bf16", "structured")
    c["3"] = RelayConfig("3", 3, 36, 8, 4, 128, 8192, 32, 1229, 8, "bf16", "structured", outlier_frac=0.01)
    c["4"] = RelayConfig("4", 4, 40, 8, 5, 128, 16384, 64, 3277, 8, "bf16", "structured", outlier_frac=0.01)
    c["5"] = RelayConfig("5", 5, 36, 8, 4, 128, 32768, 64, 0, 16, "bf16", "structured", outlier_frac=0.01,
                         budget_range=(0.099, 0.202), agents=4)
    # paper-regime shadows: budget below head_dim so the back-fill is not the identity
    c["1s"] = replace(c["1"], name="1s", budget=32)
    c["2s"] = replace(c["2"], name="2s", budget=96)
    c["3s"] = replace(c["3"], name="3s", budget=96)
    c["4s"] = replace(c["4"], name="4s", budget=96)
    c["5s"] = replace(c["5"], name="5s", budget_range=None, budget_int_range=(32, 112))
    # the shape the paper itself runs at: a few hundred prompt tokens, budget 32, rank 2
    c["paper"] = RelayConfig("paper", 6, 36, 8, 4, 128, 256, 32, 32, 2, "bf16", "structured", outlier_frac=0.01)
    return c


CONFIGS: Dict[str, RelayConfig] = _named()


def shrink(cfg: RelayConfig, *, n_layers: Optional[int] = None, n_kv_heads: Optional[int] = None,
           n_tokens: Optional[int] = None, budget: Optional[int] = None, name: Optional[str] = None,
           **kw) -> RelayConfig:
    """A smaller/other-shaped copy of a config (same distribution and seeding id)."""
    upd = dict(kw)
    if n_layers is not None:
        upd["n_layers"] = n_layers
    if n_kv_heads is not None:
        upd["n_kv_heads"] = n_kv_heads
    if n_tokens is not None:
        upd["n_tokens"] = n_tokens
    if budget is not None:
        upd["budget"] = budget
    upd["name"] = name or (cfg.name + "-shrunk")
    return replace(cfg, **upd)


# --------------------------------------------------------------------------- dtype plumbing
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def _to_io(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def io_numpy_dtype(dtype: str):
    return np.float32 if dtype == "f32" else np.uint16


# --------------------------------------------------------------------------- generators
def _rng(seed: int, cfg: RelayConfig, layer: int, head: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg.base, layer, head, tensor])))


def outlier_tokens(cfg: RelayConfig, seed: int, layer: int) -> np.ndarray:
    """Sorted outlier token indices of one layer (empty when the config has none)."""
    n = int(round(cfg.outlier_frac * cfg.n_tokens))
    if n <= 0:
        return np.zeros(0, dtype=np.int64)
    rng = _rng(seed, cfg, layer, _OUTLIER_HEAD, _T_HEAVY)
    return np.sort(rng.choice(cfg.n_tokens, size=n, replace=False))


def _structured(rng: np.random.Generator, n: int, d: int, lowrank: int) -> np.ndarray:
    e = rng.standard_normal((n, d), dtype=np.float32)
    f = rng.standard_normal((n, lowrank), dtype=np.float32)
    g = rng.standard_normal((lowrank, d), dtype=np.float32)
    z = rng.standard_normal(d, dtype=np.float32)
    s = np.exp(np.float32(0.5) * z).astype(np.float32)
    x = np.float32(np.sqrt(0.5)) * e + (f @ g) * np.float32(np.sqrt(0.5) / np.sqrt(lowrank))
    x *= s[None, :]
    return x


def head_kv(cfg: RelayConfig, seed: int, layer: int, kv_head: int) -> Tuple[np.ndarray, np.ndarray]:
    """K, V of one (layer, kv_head): arrays [n_tokens, head_dim] in the config's I/O dtype."""
    n, d = cfg.n_tokens, cfg.head_dim
    rk = _rng(seed, cfg, layer, kv_head, _T_K)
    rv = _rng(seed, cfg, layer, kv_head, _T_V)
    if cfg.dist == "iid":
        k = rk.standard_normal((n, d), dtype=np.float32)
        v = rv.standard_normal((n, d), dtype=np.float32)
        if cfg.heavy > 0:
            rh = _rng(seed, cfg, layer, kv_head, _T_HEAVY)
            rows = rh.choice(n, size=min(cfg.heavy, n), replace=False)
            k[rows, :] *= np.float32(cfg.heavy_scale)
    elif cfg.dist == "structured":
        k = _structured(rk, n, d, cfg.lowrank)
        v = _structured(rv, n, d, cfg.lowrank)
        out = outlier_tokens(cfg, seed, layer)
        if out.size:
            k[out, :] *= np.float32(cfg.outlier_scale)
            v[out, :] *= np.float32(cfg.outlier_scale)
    else:
        raise ValueError(cfg.dist)
    return _to_io(k, cfg.dtype), _to_io(v, cfg.dtype)


def head_q(cfg: RelayConfig, seed: int, layer: int, kv_head: int) -> np.ndarray:
    """Window queries of the `group` query heads that share one KV head: [group, window, head_dim]."""
    rq = _rng(seed, cfg, layer, kv_head, _T_Q)
    q = rq.standard_normal((cfg.group, cfg.window, cfg.head_dim), dtype=np.float32)
    return _to_io(q, cfg.dtype)


def budgets(cfg: RelayConfig, seed: int) -> np.ndarray:
    """Per-head budgets, int32 [n_layers, n_kv_heads]."""
    shape = (cfg.n_layers, cfg.n_kv_heads)
    if cfg.budget_range is not None:
        rng = _rng(seed, cfg, 0, 0, _T_BUDGET)
        u = rng.uniform(cfg.budget_range[0], cfg.budget_range[1], size=shape)
        return np.rint(u * cfg.n_tokens).astype(np.int32)
    if cfg.budget_int_range is not None:
        rng = _rng(seed, cfg, 0, 0, _T_BUDGET)
        lo, hi = cfg.budget_int_range
        return rng.integers(lo, hi + 1, size=shape).astype(np.int32)
    return np.full(shape, cfg.budget, dtype=np.int32)


def make_cache(cfg: RelayConfig, seed: int = 0, threads: int = 8,
               heads: Optional[Iterable[Tuple[int, int]]] = None):
    """Whole cache in the canonical layout.

    Returns (K, V, Q_win): K, V [L, H_kv, N, d]; Q_win [L, H_kv*group, W, d].
    When `heads` is given only those (layer, kv_head) slices are filled (the rest stay zero).
    """
    L, H, N, d, g, W = cfg.n_layers, cfg.n_kv_heads, cfg.n_tokens, cfg.head_dim, cfg.group, cfg.window
    dt = io_numpy_dtype(cfg.dtype)
    K = np.zeros((L, H, N, d), dtype=dt)
    V = np.zeros((L, H, N, d), dtype=dt)
    Q = np.zeros((L, H * g, W, d), dtype=dt)
    todo = list(heads) if heads is not None else [(l, h) for l in range(L) for h in range(H)]

    def work(lh):
        l, h = lh
        k, v = head_kv(cfg, seed, l, h)
        K[l, h] = k
        V[l, h] = v
        Q[l, h * g:(h + 1) * g] = head_q(cfg, seed, l, h)

    if threads <= 1 or len(todo) <= 1:
        for lh in todo:
            work(lh)
    else:
        with _cf.ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, todo))
    return K, V, Q
