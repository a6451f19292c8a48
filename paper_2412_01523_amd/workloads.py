"""Seeded synthetic workloads: packed-batch length lists and bf16 N(0,1) tensors.

This module is the only code shared by the HIP path's tests/bench and the CPU
oracle's tests.  It holds no attention or permute arithmetic: only a
counter-based random generator (numpy's Philox), the length recipes of the five
benchmark configurations, and the bf16 <-> float bit conversions needed to hand
the *same bit patterns* to both sides.

The paper measures on GitHub / CommonCrawl / Wikipedia (Sec. 6.1, "Experimental
Setups"), corpora with long-tail length distributions (Sec. 3, Fig. 3: most
sequences are short, a few are very long).  Those corpora are not available
here; the recipes below are synthetic stand-ins with the same structure.

bf16 tensors are carried on the host as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

BASE_SEED = 20241201

# tensor ids used to key the generator
TID_Q, TID_K, TID_V, TID_DO, TID_X = 0, 1, 2, 3, 4
TID_LENGTHS = 999


@dataclass(frozen=True)
class Config:
    """One benchmark configuration (shape of one GPU's share after the scatter)."""
    index: int          # 0-based index into CONFIGS
    name: str
    tokens: int         # T, total tokens in the packed batch
    hq: int             # query heads held by this GPU
    hkv: int            # KV heads held by this GPU
    d: int              # head dim
    sp_degree: int      # P used for the pack/unpack leg (0: no permute leg defined)
    causal: bool = True

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * (self.index + 1)


CONFIGS: Tuple[Config, ...] = (
    Config(0, "tiny-436", 436, 4, 4, 64, 0),
    Config(1, "lognormal-32k", 32768, 4, 4, 128, 8),
    Config(2, "pareto-64k", 65536, 8, 8, 128, 8),
    Config(3, "single-128k", 131072, 8, 8, 128, 0),
    Config(4, "bimodal-256k-gqa", 262144, 16, 2, 128, 0),
)


def _rng(seed: int, tid: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tid)]))


# --------------------------------------------------------------------------
# bf16 bit helpers (format conversion only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), return uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # NaN stays NaN (quiet); everything else: add 0x7FFF + lsb then truncate
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint32(0x7FC0), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def normal_bf16(seed: int, tid: int, shape) -> np.ndarray:
    """i.i.d. N(0,1), rounded to bf16; uint16 bit patterns of the given shape."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    g = _rng(seed, tid)
    chunk = 1 << 24
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = f32_to_bf16_bits(g.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


def index_pattern_u16(shape) -> np.ndarray:
    """A tensor whose every element encodes (a hash of) its own flat index; used by
    the permute tests so that a misplaced element cannot go unnoticed."""
    n = int(np.prod(shape))
    i = np.arange(n, dtype=np.uint64)
    h = (i * np.uint64(0x9E3779B97F4A7C15)) >> np.uint64(48)
    return h.astype(np.uint16).reshape(shape)


# --------------------------------------------------------------------------
# length recipes
# --------------------------------------------------------------------------
def _fill(draw, total: int) -> List[int]:
    """Draw lengths until `total` tokens are used; the last one is truncated to the
    remaining budget (even when that is below the recipe's lower clip)."""
    out: List[int] = []
    left = total
    while left > 0:
        s = int(draw())
        s = min(s, left)
        out.append(s)
        left -= s
    return out


def lengths(cfg: Config, seed: int | None = None) -> List[int]:
    """The realised sequence-length list of a configuration (sums to cfg.tokens)."""
    seed = cfg.seed if seed is None else seed
    g = _rng(seed, TID_LENGTHS)
    if cfg.index == 0:
        return [17, 64, 100, 255]
    if cfg.index == 1:
        def draw():
            return int(np.clip(np.rint(np.exp(g.normal(7.0, 1.2))), 128, 32768))
        return _fill(draw, cfg.tokens)
    if cfg.index == 2:
        def draw():
            u = 1.0 - g.random()          # (0, 1]
            return int(np.clip(np.floor(256.0 * u ** (-1.0 / 1.1)), 256, 65536))
        return _fill(draw, cfg.tokens)
    if cfg.index == 3:
        return [cfg.tokens]
    if cfg.index == 4:
        long = [65536, 65536, 32768]
        rest = cfg.tokens - sum(long)
        short = _fill(lambda: int(g.integers(64, 1025)), rest)
        all_ = long + short
        perm = g.permutation(len(all_))
        return [all_[i] for i in perm]
    raise ValueError("unknown config")


def cu_seqlens(lens) -> np.ndarray:
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    np.cumsum(np.asarray(lens, dtype=np.int64), out=cu[1:])
    return cu


def causal_pairs(lens) -> int:
    """Number of (query, key) pairs under the causal mask, diagonal included."""
    return int(sum(int(s) * (int(s) + 1) // 2 for s in lens))


def attn_flops(lens, hq: int, d: int, causal: bool = True) -> Tuple[int, int]:
    """(forward, backward) FLOPs in the causal-effective convention: two GEMMs
    forward, five backward, 2 FLOP per MAC, masked pairs not counted."""
    pairs = causal_pairs(lens) if causal else int(sum(int(s) * int(s) for s in lens))
    fwd = 4 * d * hq * pairs
    return fwd, fwd * 5 // 2


def make_qkvdo(cfg: Config, tokens: int | None = None, seed: int | None = None):
    """q [T,Hq,D], k,v [T,Hkv,D], dO [T,Hq,D] as bf16 bit patterns (uint16)."""
    t = cfg.tokens if tokens is None else tokens
    seed = cfg.seed if seed is None else seed
    q = normal_bf16(seed, TID_Q, (t, cfg.hq, cfg.d))
    k = normal_bf16(seed, TID_K, (t, cfg.hkv, cfg.d))
    v = normal_bf16(seed, TID_V, (t, cfg.hkv, cfg.d))
    do = normal_bf16(seed, TID_DO, (t, cfg.hq, cfg.d))
    return q, k, v, do
