"""Seeded synthetic workloads shaped like the paper's data sets.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds no arithmetic of the method itself (no distances, no
assignment, no top-k): it only draws numbers.  Everything is a pure function of
its arguments, so both sides consume identical bits.

The paper evaluates on a 128-dimensional byte-valued public benchmark set and
on a 64-dimensional industrial embedding set (Experiment section, first
paragraph); neither is available here, so Gaussian mixtures with the same
dimension, order of magnitude and value type stand in for them.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SEED_BASE = 240802937


@dataclass
class Workload:
    """One synthetic workload: base set, centroids, queries and insert stream."""

    name: str
    metric: str  # "l2" or "ip"
    d: int
    nlist: int
    block_vecs: int  # T_m
    nprobe: int
    k: int
    base: np.ndarray  # [N][d] float32
    centroids: np.ndarray  # [nlist][d] float32
    queries: np.ndarray  # [nq][d] float32
    inserts: np.ndarray  # [ni][d] float32
    insert_batch: int
    seed: int
    extra: dict = field(default_factory=dict)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


# Sets above this many coordinates are drawn in chunks of rows, every chunk from a generator of its
# own (seeded from the parent stream), on several threads: the result is a pure function of the seed
# whatever the thread count, and a 20 GB set takes seconds instead of a minute.  Smaller sets keep
# the single-stream draw.
_BIG_SET = 1 << 27
_CHUNK_ROWS = 1 << 17


def mixture(
    rng: np.random.Generator,
    centres: np.ndarray,
    n: int,
    sigma: float,
    component: Optional[np.ndarray] = None,
    post=None,
) -> np.ndarray:
    """n points: a uniformly drawn (or given) centre plus isotropic noise.  `post`, if given,
    rewrites rows in place (rounding, normalisation)."""
    if component is None:
        component = rng.integers(0, centres.shape[0], size=n)
    d = centres.shape[1]
    if n * d <= _BIG_SET:
        out = rng.standard_normal((n, d), dtype=np.float32)
        out *= np.float32(sigma)
        out += centres[component]
        if post is not None:
            post(out)
        return out
    out = np.empty((n, d), dtype=np.float32)
    nchunks = (n + _CHUNK_ROWS - 1) // _CHUNK_ROWS
    seeds = rng.integers(0, 1 << 62, size=nchunks)

    def draw(c: int) -> None:
        r = np.random.Generator(np.random.PCG64(int(seeds[c])))
        blk = out[c * _CHUNK_ROWS:(c + 1) * _CHUNK_ROWS]
        r.standard_normal(out=blk, dtype=np.float32)
        blk *= np.float32(sigma)
        blk += centres[component[c * _CHUNK_ROWS:(c + 1) * _CHUNK_ROWS]]
        if post is not None:
            post(blk)

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        list(pool.map(draw, range(nchunks)))
    return out


def _unit_rows(x: np.ndarray) -> None:
    """Rows scaled to unit length in place (norm in double, one rounding to float)."""
    nrm = np.sqrt((x.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
    x[:] = (x / np.maximum(nrm, 1e-30)).astype(np.float32)


def _pick_rows(rng: np.random.Generator, base: np.ndarray, n: int) -> np.ndarray:
    """n distinct rows of base chosen by a seeded permutation."""
    idx = rng.permutation(base.shape[0])[:n]
    return np.ascontiguousarray(base[idx])


def gaussian_l2(
    name: str,
    seed: int,
    d: int = 32,
    n_base: int = 10_000,
    n_centres: int = 100,
    sigma: float = 0.1,
    nlist: int = 64,
    block_vecs: int = 64,
    n_queries: int = 1_000,
    n_inserts: int = 1_000,
    insert_batch: int = 100,
    nprobe: int = 8,
    k: int = 10,
) -> Workload:
    """Small real-valued L2 workload (the tiny parity configuration)."""
    centres = _rng(seed, 0).standard_normal((n_centres, d), dtype=np.float32)
    base = mixture(_rng(seed, 1), centres, n_base, sigma)
    centroids = _pick_rows(_rng(seed, 2), base, nlist)
    queries = mixture(_rng(seed, 3), centres, n_queries, sigma)
    inserts = mixture(_rng(seed, 4), centres, n_inserts, sigma)
    return Workload(name, "l2", d, nlist, block_vecs, nprobe, k, base, centroids,
                    queries, inserts, insert_batch, seed)


def byte_valued_l2(
    name: str,
    seed: int,
    d: int = 128,
    n_base: int = 1_000_000,
    n_centres: int = 1_000,
    sigma: float = 20.0,
    nlist: int = 1024,
    block_vecs: int = 128,
    n_queries: int = 10_000,
    n_inserts: int = 100_000,
    insert_batch: int = 64,
    nprobe: int = 32,
    k: int = 100,
) -> Workload:
    """fp32 vectors holding integers 0..255: centres ~ U(0,128) per coordinate,
    Gaussian noise, rounded and clipped."""
    centres = _rng(seed, 0).uniform(0.0, 128.0, size=(n_centres, d)).astype(np.float32)

    def to_bytes(x: np.ndarray) -> None:
        np.rint(x, out=x)
        np.clip(x, 0.0, 255.0, out=x)

    def draw(stream: int, n: int) -> np.ndarray:
        return mixture(_rng(seed, stream), centres, n, sigma, post=to_bytes)

    base = draw(1, n_base)
    centroids = _pick_rows(_rng(seed, 2), base, nlist)
    queries = draw(3, n_queries)
    inserts = draw(4, n_inserts)
    return Workload(name, "l2", d, nlist, block_vecs, nprobe, k, base, centroids,
                    queries, inserts, insert_batch, seed)


def unit_ip(
    name: str,
    seed: int,
    d: int = 96,
    n_base: int = 100_000,
    n_centres: int = 1_000,
    sigma: float = 0.1,
    nlist: int = 256,
    block_vecs: int = 256,
    n_queries: int = 1_000,
    n_inserts: int = 4_096,
    insert_batch: int = 512,
    nprobe: int = 16,
    k: int = 10,
) -> Workload:
    """Unit-normalised embeddings searched by inner product."""
    centres = _rng(seed, 0).standard_normal((n_centres, d), dtype=np.float32)
    base = mixture(_rng(seed, 1), centres, n_base, sigma, post=_unit_rows)
    centroids = _pick_rows(_rng(seed, 2), base, nlist)
    queries = mixture(_rng(seed, 3), centres, n_queries, sigma, post=_unit_rows)
    inserts = mixture(_rng(seed, 4), centres, n_inserts, sigma, post=_unit_rows)
    return Workload(name, "ip", d, nlist, block_vecs, nprobe, k, base, centroids,
                    queries, inserts, insert_batch, seed)


def zipf_lists(n_lists: int, n: int, exponent: float, rng: np.random.Generator) -> np.ndarray:
    """n list indices whose popularity follows a truncated Zipf law over a
    seeded permutation of the lists."""
    w = 1.0 / np.arange(1, n_lists + 1, dtype=np.float64) ** exponent
    w /= w.sum()
    rank_of = rng.permutation(n_lists)
    return rank_of[rng.choice(n_lists, size=n, p=w)]


def skewed_l2(
    name: str,
    seed: int,
    d: int = 64,
    n_base: int = 200_000,
    nlist: int = 512,
    exponent: float = 1.1,
    sigma: float = 0.1,
    block_vecs: int = 64,
    n_queries: int = 512,
    n_inserts: int = 8_192,
    insert_batch: int = 1024,
    nprobe: int = 16,
    k: int = 50,
) -> Workload:
    """Skewed growth: the centroids are the mixture centres and the component of
    each point follows a Zipf law, so a few hot lists grow by many blocks."""
    centroids = _rng(seed, 0).standard_normal((nlist, d), dtype=np.float32)

    # one ranking for every stream: draw it once and reuse
    ranking = _rng(seed, 100).permutation(nlist)
    w = 1.0 / np.arange(1, nlist + 1, dtype=np.float64) ** exponent
    w /= w.sum()

    def draw_ranked(stream: int, n: int):
        r = _rng(seed, stream)
        comp = ranking[r.choice(nlist, size=n, p=w)]
        return mixture(r, centroids, n, sigma, component=comp), comp

    base, base_comp = draw_ranked(1, n_base)
    queries, _ = draw_ranked(3, n_queries)
    inserts, ins_comp = draw_ranked(4, n_inserts)
    return Workload(name, "l2", d, nlist, block_vecs, nprobe, k, base, centroids,
                    queries, inserts, insert_batch, seed,
                    extra={"base_component": base_comp, "insert_component": ins_comp,
                           "ranking": ranking})


def config(idx: int, scale: float = 1.0) -> Workload:
    """The benchmark configurations, by number.  `scale` < 1 shrinks the base,
    query and insert counts (never d, nlist, T_m, nprobe or k) for quick runs."""
    s = lambda n: max(1, int(round(n * scale)))
    seed = SEED_BASE + idx
    if idx == 1:
        return gaussian_l2("config1-tiny-l2", seed, n_base=s(10_000), n_queries=s(1_000),
                           n_inserts=s(1_000))
    if idx == 2:
        return byte_valued_l2("config2-byte-l2-d128", seed, n_base=s(1_000_000),
                              n_queries=s(10_000), n_inserts=s(100_000))
    if idx == 3:
        return unit_ip("config3-unit-ip-d96", seed, d=96, n_base=s(10_000_000),
                       n_centres=10_000, nlist=4096, block_vecs=256, n_queries=s(10_000),
                       n_inserts=s(500_000), insert_batch=512, nprobe=64, k=10)
    if idx == 4:
        return unit_ip("config4-unit-ip-d768", seed, d=768, n_base=s(5_000_000),
                       n_centres=10_000, nlist=8192, block_vecs=128, n_queries=s(4_096),
                       n_inserts=s(65_536), insert_batch=64, nprobe=32, k=10)
    if idx == 5:
        return skewed_l2("config5-zipf-l2-d256", seed, d=256, n_base=s(20_000_000),
                         nlist=16384, block_vecs=256, n_queries=s(4_096),
                         n_inserts=s(1_000_000), insert_batch=1024, nprobe=64, k=50)
    raise ValueError(f"no such configuration: {idx}")


def codebooks_from_rows(seed: int, rows: np.ndarray, m: int) -> np.ndarray:
    """Codebooks [m][256][d/m] for product-quantised lists: entry c of sub-space s
    is sub-vector s of a row drawn by a seeded permutation (256 distinct rows per
    sub-space).  A stand-in for trained codebooks: training is outside the path."""
    d = rows.shape[1]
    ds = d // m
    out = np.empty((m, 256, ds), dtype=np.float32)
    for s in range(m):
        idx = _rng(seed, 200 + s).permutation(rows.shape[0])[:256]
        out[s] = rows[idx, s * ds:(s + 1) * ds]
    return out
