"""Seeded synthetic workloads for the D-CHAG tokenize + hierarchical-aggregate path.

This module only draws random numbers and shapes them: it holds none of the
method's arithmetic.  Both the CPU oracle and the HIP path read the arrays it
returns; neither of them is imported here.

Shapes follow the paper's two application domains (Section 5): weather
reanalysis with about 80 variables on a lat-lon grid, and plant hyperspectral
images with about 500 contiguous bands.  The data themselves are not
available, so only their channel counts and rough statistics are borrowed.

Every array is float32.  For a bf16 run every value is first rounded once to
bf16 (round-to-nearest-even) and stored back as float32, so that the oracle
(which widens to fp64) and the GPU path (which narrows to bf16, exactly) read
the same numbers.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

__all__ = [
    "ShapeCfg", "Level", "Problem", "CONFIGS", "get_config", "n_groups", "make_level", "make_linear_level",
    "level_inputs", "round_to_bf16", "make_problem", "make_tokens", "sample_patches", "sample_patches_covering",
]


@dataclass(frozen=True)
class ShapeCfg:
    name: str
    dtype: str                     # "f32" | "bf16"
    B: int
    C: int
    H: int
    W: int
    p: int
    D: int
    heads: int
    group_sizes: Sequence[int]     # nominal group size per level, last level must give one group
    x_kind: str = "gauss"          # "gauss_mu_sigma" | "weather" | "ar1" | "gauss"
    seed: int = 0
    level_kinds: Optional[Sequence[str]] = None   # per level "attention" (default) or "linear" (D-CHAG-L)

    @property
    def N(self) -> int:
        return (self.H // self.p) * (self.W // self.p)

    @property
    def tokens(self) -> int:
        return self.B * self.C * self.N


def n_groups(c_in: int, g: int) -> int:
    """Number of contiguous groups of nominal size g covering c_in members (last may be short)."""
    return (c_in + g - 1) // g


def level_inputs(C: int, group_sizes: Sequence[int]) -> List[int]:
    """Number of input tokens per patch at each level (C, G_1, G_2, ...)."""
    out = [C]
    for g in group_sizes:
        out.append(n_groups(out[-1], g))
    return out[:-1]


CONFIGS = {
    "tiny": ShapeCfg("tiny", "f32", 1, 8, 32, 64, 4, 128, 4, (4, 2), "gauss_mu_sigma", 0),
    "weather": ShapeCfg("weather", "bf16", 2, 80, 128, 256, 4, 1024, 16, (8, 10), "weather", 1),
    "hyperspectral": ShapeCfg("hyperspectral", "bf16", 4, 512, 128, 128, 8, 1024, 16, (32, 16), "ar1", 2),
    "wide": ShapeCfg("wide", "bf16", 1, 256, 256, 512, 8, 4096, 32, (32, 8), "gauss", 3),
    "deep": ShapeCfg("deep", "bf16", 2, 1024, 128, 128, 8, 2048, 16, (16, 8, 8), "ar1", 4),
    "deep1000": ShapeCfg("deep1000", "bf16", 2, 1000, 128, 128, 8, 2048, 16, (16, 8, 8), "ar1", 4),
    # the flat baseline the hierarchy is compared with (Sections 2.1, 3.2): one cross-attention layer over all channels
    "hyperspectral_flat": ShapeCfg("hyperspectral_flat", "bf16", 4, 512, 128, 128, 8, 1024, 16, (512,), "ar1", 2),
    # D-CHAG-L (Section 4.5): linear partial-aggregation layers, cross-attention only at the top
    "hyperspectral_linear": ShapeCfg("hyperspectral_linear", "bf16", 4, 512, 128, 128, 8, 1024, 16, (32, 16), "ar1", 2,
                                     ("linear", "attention")),
}


def get_config(name: str) -> ShapeCfg:
    return CONFIGS[name]


_BLOCK = 1 << 22                       # elements per block of the block-parallel paths below
_THREADS = max(1, min(16, os.cpu_count() or 1))


def _for_blocks(n: int, fn) -> None:
    """fn(lo, hi) over the blocks of range(n), on a few threads for large n (numpy releases the GIL in these loops);
    the result does not depend on the number of threads."""
    spans = [(i, min(n, i + _BLOCK)) for i in range(0, n, _BLOCK)]
    if len(spans) <= 1 or _THREADS == 1:
        for lo, hi in spans:
            fn(lo, hi)
        return
    with ThreadPoolExecutor(_THREADS) as ex:
        list(ex.map(lambda sp: fn(*sp), spans))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty_like(a)
    src, dst = a.reshape(-1).view(np.uint32), out.reshape(-1).view(np.uint32)

    def block(lo, hi):
        u = src[lo:hi]
        r = (u >> np.uint32(16)) & np.uint32(1)
        r += np.uint32(0x7FFF)
        r += u                                         # finite inputs only: no carry out of 32 bits
        r &= np.uint32(0xFFFF0000)
        dst[lo:hi] = r

    _for_blocks(src.size, block)
    return out


@dataclass
class Level:
    group_size: int
    query: Optional[np.ndarray]    # [G, D]
    Wq: Optional[np.ndarray]       # [G, D, D]  (out, in)
    Wk: Optional[np.ndarray]
    Wv: np.ndarray                 # attention: [G, D, D]; linear: channel-mixing weights [G, g, D]
    Wo: Optional[np.ndarray]
    bq: Optional[np.ndarray]       # [G, D] or None
    bk: Optional[np.ndarray]
    bv: Optional[np.ndarray]       # attention: value bias; linear: output bias
    bo: Optional[np.ndarray]
    kind: str = "attention"        # "attention" | "linear"

    @property
    def G(self) -> int:
        return self.Wv.shape[0]


@dataclass
class Problem:
    cfg: ShapeCfg
    x: np.ndarray                  # [B, C, H, W]
    We: np.ndarray                 # [C, D, p*p]
    be: Optional[np.ndarray]       # [C, D]
    ce: Optional[np.ndarray]       # [C, D]
    levels: List[Level] = field(default_factory=list)


def _normal(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    """N(0, std^2) float32 values.  Tensors of up to one block come straight from `rng`; a larger one takes ONE
    63-bit draw from `rng` as its key and fills block i from PCG64([key, i]), so its blocks can be drawn on several
    threads (the values depend on the seed alone, never on the number of threads)."""
    n = int(np.prod(shape))
    if n <= _BLOCK:
        a = rng.standard_normal(shape, dtype=np.float32)
        if std != 1.0:
            a *= np.float32(std)
        return a
    key = int(rng.integers(0, 2 ** 63 - 1))
    flat = np.empty(n, dtype=np.float32)

    def block(lo, hi):
        g = np.random.Generator(np.random.PCG64([key, lo // _BLOCK]))
        g.standard_normal(out=flat[lo:hi], dtype=np.float32)
        if std != 1.0:
            flat[lo:hi] *= np.float32(std)

    _for_blocks(n, block)
    return flat.reshape(shape)


def _box5(f: np.ndarray) -> np.ndarray:
    """5x5 box mean over the last two axes with wrap-around (periodic in longitude is fine here)."""
    acc = np.zeros_like(f)
    for dy in range(-2, 3):
        for dx in range(-2, 3):
            acc += np.roll(np.roll(f, dy, axis=-2), dx, axis=-1)
    return acc / 25.0


def _make_x(cfg: ShapeCfg, rng: np.random.Generator) -> np.ndarray:
    B, C, H, W = cfg.B, cfg.C, cfg.H, cfg.W
    if cfg.x_kind == "gauss_mu_sigma":
        mu = rng.uniform(-1.0, 1.0, size=C).astype(np.float32)
        sg = rng.uniform(0.5, 2.0, size=C).astype(np.float32)
        x = _normal(rng, (B, C, H, W)) * sg[None, :, None, None] + mu[None, :, None, None]
    elif cfg.x_kind == "weather":
        x = _box5(_normal(rng, (B, C, H, W)))
        x -= x.mean(axis=(0, 2, 3), keepdims=True)
        x /= x.std(axis=(0, 2, 3), keepdims=True)
        sc = rng.uniform(0.5, 2.0, size=C).astype(np.float32)
        x *= sc[None, :, None, None]
    elif cfg.x_kind == "ar1":
        rho = np.float32(0.95)
        inn = np.float32(np.sqrt(1.0 - 0.95 ** 2))
        x = np.empty((B, C, H, W), dtype=np.float32)
        prev = _normal(rng, (B, H, W))
        x[:, 0] = prev
        for c in range(1, C):
            prev = rho * prev + inn * _normal(rng, (B, H, W))
            x[:, c] = prev
        x += _normal(rng, (B, C, H, W), 0.1)
    elif cfg.x_kind == "gauss":
        x = _normal(rng, (B, C, H, W))
    else:
        raise ValueError(f"unknown x_kind {cfg.x_kind!r}")
    return np.ascontiguousarray(x, dtype=np.float32)


def make_linear_level(rng: np.random.Generator, G: int, g: int, D: int, dtype: str, biases: bool = True) -> Level:
    """A linear (D-CHAG-L) level: mixing weights around the plain mean, N(1/g, 1/g^2), bias N(0, 1/g)."""
    w = _normal(rng, (G, g, D), 1.0 / g) + np.float32(1.0 / g)
    b = _normal(rng, (G, D), 1.0 / np.sqrt(g)) if biases else None
    if dtype == "bf16":
        w = round_to_bf16(w)
        b = round_to_bf16(b) if b is not None else None
    return Level(g, None, None, None, w, None, None, None, b, None, "linear")


def make_level(rng: np.random.Generator, G: int, g: int, D: int, dtype: str,
               biases: bool = True, query_scale: float = 1.0) -> Level:
    fin = 1.0 / np.sqrt(D)

    def fin_arr(shape):
        return _normal(rng, shape, fin)

    lv = Level(
        group_size=g,
        query=_normal(rng, (G, D), query_scale),
        Wq=fin_arr((G, D, D)), Wk=fin_arr((G, D, D)), Wv=fin_arr((G, D, D)), Wo=fin_arr((G, D, D)),
        bq=fin_arr((G, D)) if biases else None,
        bk=fin_arr((G, D)) if biases else None,
        bv=fin_arr((G, D)) if biases else None,
        bo=fin_arr((G, D)) if biases else None,
    )
    if dtype == "bf16":
        for k in ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo"):
            v = getattr(lv, k)
            if v is not None:
                setattr(lv, k, round_to_bf16(v))
    return lv


def make_problem(cfg: ShapeCfg, seed: Optional[int] = None, biases: bool = True,
                 query_scale: float = 1.0, with_x: bool = True) -> Problem:
    """All inputs and weights of one forward pass, drawn from PCG64(seed).

    Weight matrices are N(0, 1/fan_in) (fan_in = p*p for the tokenizer, D for the
    attention projections); queries and channel embeddings are N(0, 1); biases,
    when present, are N(0, 1/fan_in).
    """
    seed = cfg.seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    pp = cfg.p * cfg.p
    x = _make_x(cfg, rng) if with_x else np.zeros((cfg.B, cfg.C, cfg.H, cfg.W), np.float32)
    We = _normal(rng, (cfg.C, cfg.D, pp), 1.0 / np.sqrt(pp))
    be = _normal(rng, (cfg.C, cfg.D), 1.0 / np.sqrt(pp)) if biases else None
    ce = _normal(rng, (cfg.C, cfg.D))
    if cfg.dtype == "bf16":
        x, We, ce = round_to_bf16(x), round_to_bf16(We), round_to_bf16(ce)
        be = round_to_bf16(be) if be is not None else None
    prob = Problem(cfg, x, We, be, ce)
    c_in = cfg.C
    for li, g in enumerate(cfg.group_sizes):
        G = n_groups(c_in, g)
        kind = cfg.level_kinds[li] if cfg.level_kinds else "attention"
        if kind == "linear":
            prob.levels.append(make_linear_level(rng, G, g, cfg.D, cfg.dtype, biases))
        else:
            prob.levels.append(make_level(rng, G, g, cfg.D, cfg.dtype, biases, query_scale))
        c_in = G
    if c_in != 1:
        raise ValueError("last level must reduce to one group")
    return prob


def make_tokens(B: int, Cin: int, N: int, D: int, dtype: str, seed: int) -> np.ndarray:
    """A [B, Cin, N, D] token tensor with N(0, 2) entries (the spread level-1 tokens have)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    z = _normal(rng, (B, Cin, N, D), np.sqrt(2.0))
    return round_to_bf16(z) if dtype == "bf16" else z


def sample_patches(B: int, N: int, per_batch: int, seed: int):
    """A seeded sample of patches: per_batch distinct patch indices for every batch item.

    Returns two int32 arrays (b, n) of length B*per_batch.  The first and the
    last patch of every batch item are always included when per_batch >= 2.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    bs, ns = [], []
    for b in range(B):
        k = min(per_batch, N)
        pick = set()
        if k >= 2:
            pick.update((0, N - 1))
        while len(pick) < k:
            pick.add(int(rng.integers(0, N)))
        for n in sorted(pick):
            bs.append(b)
            ns.append(n)
    return np.asarray(bs, dtype=np.int32), np.asarray(ns, dtype=np.int32)


def sample_patches_covering(B: int, N: int, per_batch: int, seed: int, tile: int = 32):
    """A seeded sample of per_batch patches per batch item that is spread over the kernels' tiling: every batch item
    gets its first and last patch and the seams of the 32- and 128-patch tiles (31, 32, 127, 128); the rest walks
    through the residues modulo `tile` in a seeded order while cycling over the tiles, so that with
    B * per_batch >= tile + 6 * B every position inside a tile and every tile of the patch axis is hit somewhere in the
    sample.  Returns two int32 arrays (b, n), sorted by (b, n)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    ntile = (N + tile - 1) // tile
    want = min(per_batch, N)
    forced = [n for n in (0, N - 1, tile - 1, tile, 4 * tile - 1, 4 * tile) if 0 <= n < N]
    picks = [set(forced[:want]) for _ in range(B)]
    order = [int(r) for r in rng.permutation(tile)]
    i = 0
    while any(len(p) < want for p in picks):
        n = ((i * 3 + i // tile) % ntile) * tile + order[i % tile]
        i += 1
        if n >= N:
            continue
        b = min(range(B), key=lambda q: (len(picks[q]), q))
        picks[b].add(n)
    bs, ns = [], []
    for b in range(B):
        for n in sorted(picks[b]):
            bs.append(b)
            ns.append(n)
    return np.asarray(bs, dtype=np.int32), np.asarray(ns, dtype=np.int32)
