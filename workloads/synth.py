"""Seeded tensor generators.

Every tensor gets its own ``numpy.random.Generator(PCG64(seed))`` with the seed
derived from (config name, base seed, layer, tensor name, expert), so any single
tensor can be regenerated alone and in any order.

Storage dtypes
--------------
* ``f32`` configs: ``numpy.float32`` arrays.
* ``bf16`` configs: values are drawn in float32 and rounded ONCE, round to
  nearest even, to bfloat16; the arrays returned are ``numpy.uint16`` bit
  patterns.  Both consumers (the CPU oracle and the GPU library) start from
  these same bits; each widens them with its own code.

Layouts (row-major, logical):
  X  [T, H]        hidden states, N(0, 1)
  Wr [E, H]        router weights, N(0, w_std)
  b  [E] float32   router bias (never rounded to bf16)
  Wg [E+S, F, H]   gate projections, routed experts first then shared experts
  Wu [E+S, F, H]   up projections
  Wd [E+S, H, F]   down projections
"""
from __future__ import annotations

import hashlib
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import MoEConfig


def tensor_seed(cfg: MoEConfig, layer: int, name: str, expert: int = -1,
                step: int = -1) -> int:
    key = f"{cfg.name}|{cfg.seed}|{layer}|{name}|{expert}|{step}".encode()
    return int.from_bytes(hashlib.blake2b(key, digest_size=8).digest(), "little")


def _rng(cfg, layer, name, expert=-1, step=-1):
    return np.random.Generator(np.random.PCG64(tensor_seed(cfg, layer, name, expert, step)))


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest even); return uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    if np.isnan(a).any():
        raise ValueError("generator produced NaN")
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + (np.uint32(0x7FFF) + lsb)
    return (r >> np.uint32(16)).astype(np.uint16)


def _store(cfg: MoEConfig, a: np.ndarray) -> np.ndarray:
    return a if cfg.dtype == "f32" else bf16_bits_from_f32(a)


def _normal(cfg, layer, name, shape, std, expert=-1, step=-1):
    g = _rng(cfg, layer, name, expert, step)
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def make_hidden(cfg: MoEConfig, step: int = 0, T: int | None = None) -> np.ndarray:
    """X [T, H] ~ N(0,1) in the storage dtype.  Each decode step is an
    independent batch (its own seed)."""
    T = cfg.T if T is None else T
    return _store(cfg, _normal(cfg, 0, "X", (T, cfg.H), 1.0, step=step))


def make_router(cfg: MoEConfig, layer: int = 0):
    """(Wr [E,H] storage dtype, b [E] float32)."""
    Wr = _store(cfg, _normal(cfg, layer, "Wr", (cfg.E, cfg.H), cfg.w_std))
    if cfg.bias == "none":
        b = np.zeros(cfg.E, dtype=np.float32)
    elif cfg.bias == "normal":
        b = _normal(cfg, layer, "b", (cfg.E,), cfg.bias_scale)
    elif cfg.bias == "zipf":
        # The popularity prior over experts is Zipf(s): expert with (seeded,
        # random) rank r gets log-prior  ln(r^-s / sum_r r^-s).
        g = _rng(cfg, layer, "b")
        rank = g.permutation(cfg.E).astype(np.float64) + 1.0
        p = rank ** (-cfg.bias_scale)
        b = np.log(p / p.sum()).astype(np.float32)
    else:
        raise ValueError(cfg.bias)
    return Wr, b


def make_expert(cfg: MoEConfig, layer: int, e: int):
    """(Wg [F,H], Wu [F,H], Wd [H,F]) of expert ``e`` (e >= E: shared expert)."""
    Wg = _store(cfg, _normal(cfg, layer, "Wg", (cfg.F, cfg.H), cfg.w_std, expert=e))
    Wu = _store(cfg, _normal(cfg, layer, "Wu", (cfg.F, cfg.H), cfg.w_std, expert=e))
    Wd = _store(cfg, _normal(cfg, layer, "Wd", (cfg.H, cfg.F), cfg.w_std, expert=e))
    return Wg, Wu, Wd


def make_layer(cfg: MoEConfig, layer: int = 0, step: int = 0, threads: int = 8,
               with_hidden: bool = True) -> dict:
    """All tensors of one layer.  Expert matrices are stacked [E+S, ...]."""
    n = cfg.E + cfg.S
    st = np.float32 if cfg.dtype == "f32" else np.uint16
    Wg = np.empty((n, cfg.F, cfg.H), dtype=st)
    Wu = np.empty((n, cfg.F, cfg.H), dtype=st)
    Wd = np.empty((n, cfg.H, cfg.F), dtype=st)

    def fill(e):
        Wg[e], Wu[e], Wd[e] = make_expert(cfg, layer, e)

    if threads > 1 and n > 1:
        with ThreadPoolExecutor(max_workers=min(threads, n)) as ex:
            list(ex.map(fill, range(n)))
    else:
        for e in range(n):
            fill(e)
    Wr, b = make_router(cfg, layer)
    out = {"Wr": Wr, "b": b, "Wg": Wg, "Wu": Wu, "Wd": Wd}
    if with_hidden:
        out["X"] = make_hidden(cfg, step)
    return out


def make_residency_mask(cfg: MoEConfig, layer: int, n_resident: int | None = None) -> np.ndarray:
    """bool [E]: which routed experts of ``layer`` start out in device memory
    (seeded choice of ``n_resident`` of E; default half)."""
    n_resident = cfg.E // 2 if n_resident is None else n_resident
    g = _rng(cfg, layer, "resident")
    m = np.zeros(cfg.E, dtype=bool)
    m[g.choice(cfg.E, size=n_resident, replace=False)] = True
    return m


def make_prefetch_noise(cfg: MoEConfig, layer: int, step: int, std: float = 0.5) -> np.ndarray:
    """float32 [T, E] noise a harness adds to the NEXT layer's router logits to
    imitate an imperfect expert predictor."""
    return _normal(cfg, layer, "prefetch_noise", (cfg.T, cfg.E), std, step=step)
