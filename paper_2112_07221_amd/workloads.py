"""Seeded synthetic inputs for the embedding-cache step.

This module only draws random inputs (ID streams, gradients, table initial values) and names
the workload configurations.  It contains none of the cache method's arithmetic, so both the
CPU oracle's tests and the HIP path's tests may read the same arrays from it.

The paper evaluates on click-through and graph datasets whose embedding-update frequencies
follow a power law (Section 2.3, Figure 3: the most popular tenth of the embeddings receives
about nine tenths of the updates).  Those datasets are not used here; the streams below keep
only that shape: categorical fields with finite-support Zipf popularity.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

LRU, LFU, LFU_LIGHT = 0, 1, 3
SGD, ADAGRAD, ADAGRAD_ROWWISE = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration.  `layout` is how a batch's IDs are drawn:
    "fields": `batch` samples x `width` fields, field f owns the f-th of `width` disjoint ranges;
    "flat":   `batch` x `width` IDs i.i.d. from one Zipf over the whole vocabulary;
    "bags":   `batch` bags of `width` IDs each (pooled lookup), one Zipf over the vocabulary."""
    index: int
    name: str
    vocab: int
    dim: int
    batch: int
    width: int
    layout: str
    alpha: float
    capacity: int
    policy: int
    s: int
    optimizer: int
    lr: float
    eps: float
    iters: int
    backing: str = "hbm"        # "hbm" or "host" (pinned host DRAM)
    grad_pool: int = 8

    @property
    def n(self) -> int:
        return self.batch * self.width

    @property
    def pooled(self) -> bool:
        return self.layout == "bags"

    @property
    def n_grad_rows(self) -> int:
        return self.batch if self.pooled else self.n

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    1: Workload(1, "tiny", 10_000, 16, 128, 26, "fields", 1.1, 1_000, LRU, 10, SGD, 0.01, 0.0, 100),
    2: Workload(2, "1M-ID", 1_000_000, 64, 4_096, 26, "fields", 1.05, 100_000, LFU, 100, ADAGRAD,
                0.01, 1e-8, 1_000),
    3: Workload(3, "host-backed-33M", 33_000_000, 128, 8_192, 26, "fields", 1.05, 2_000_000, LRU,
                100, SGD, 0.01, 0.0, 300, backing="host"),
    4: Workload(4, "skip-gram", 4_000_000, 128, 16_384, 7, "flat", 0.9, 400_000, LFU, 50, SGD,
                0.025, 0.0, 300),
    5: Workload(5, "bag-of-words", 1_000_000, 256, 2_048, 200, "bags", 1.0, 50_000, LFU, 100,
                ADAGRAD, 0.01, 1e-8, 300),
}


def seeds(index: int) -> dict:
    return {"table": 1000 + index, "ids": 2000 + index, "grads": 3000 + index,
            "perm": 4000 + index}


def _zipf_cdf(n: int, alpha: float) -> np.ndarray:
    """Cumulative distribution of p_r ~ r^-alpha on ranks r = 1..n, in fp64."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-alpha)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    cdf[-1] = 1.0
    return cdf


class IdStream:
    """Draws batches of int64 IDs for a workload.  Rank r of a range maps to
    `lo + perm[r]`, with `perm` a seeded permutation (popular rows are scattered over the
    range, as hashed categorical IDs are) unless `identity_perm` is set."""

    def __init__(self, wl: Workload, identity_perm: bool = False, seed: Optional[int] = None):
        self.wl = wl
        sd = seeds(wl.index)
        self.rng = np.random.Generator(np.random.PCG64(sd["ids"] if seed is None else seed))
        prng = np.random.Generator(np.random.PCG64(sd["perm"]))
        if wl.layout == "fields":
            bounds = [(f * wl.vocab) // wl.width for f in range(wl.width + 1)]
        else:
            bounds = [0, wl.vocab]
        self.lo = np.asarray(bounds[:-1], dtype=np.int64)
        sizes = np.diff(np.asarray(bounds, dtype=np.int64))
        if np.any(sizes <= 0):
            raise ValueError("every ID range needs at least one ID")
        cdf_cache = {}
        self.cdfs, self.perms = [], []
        for sz in sizes.tolist():
            if sz not in cdf_cache:
                cdf_cache[sz] = _zipf_cdf(sz, wl.alpha)
            self.cdfs.append(cdf_cache[sz])
            self.perms.append(np.arange(sz, dtype=np.int64) if identity_perm
                              else prng.permutation(sz).astype(np.int64))

    def batches(self, iters: int) -> np.ndarray:
        """Returns ids[iters, n] int64; within an iteration the layout is [batch][width]."""
        wl = self.wl
        out = np.empty((iters, wl.batch, wl.width), dtype=np.int64)
        if wl.layout == "fields":
            for f in range(wl.width):
                u = self.rng.random((iters, wl.batch))
                r = np.minimum(np.searchsorted(self.cdfs[f], u, side="right"),
                               len(self.cdfs[f]) - 1)
                out[:, :, f] = self.lo[f] + self.perms[f][r]
        else:
            u = self.rng.random((iters, wl.batch, wl.width))
            r = np.minimum(np.searchsorted(self.cdfs[0], u, side="right"), len(self.cdfs[0]) - 1)
            out[:] = self.perms[0][r]
        return out.reshape(iters, wl.n)


def bag_offsets(wl: Workload) -> np.ndarray:
    """offsets[batch+1] int64 for the pooled layout: bag b holds ids[offsets[b]:offsets[b+1]]."""
    return np.arange(wl.batch + 1, dtype=np.int64) * wl.width


def grad_pool(wl: Workload, seed: Optional[int] = None) -> np.ndarray:
    """grads[pool, rows, dim] fp32 ~ N(0,1); iteration t uses grads[t % pool].  `rows` is one per
    lookup, or one per bag for the pooled layout."""
    rng = np.random.Generator(np.random.PCG64(seeds(wl.index)["grads"] if seed is None else seed))
    return rng.standard_normal((wl.grad_pool, wl.n_grad_rows, wl.dim), dtype=np.float32)


def table_init(wl: Workload, seed: Optional[int] = None, tile_rows: int = 1 << 20) -> np.ndarray:
    """table[vocab, dim] fp32 ~ N(0, std 0.01).  Tables above `tile_rows` rows repeat a seeded
    block of `tile_rows` rows (the values carry no meaning; this bounds generation time)."""
    rng = np.random.Generator(np.random.PCG64(seeds(wl.index)["table"] if seed is None else seed))
    rows = min(wl.vocab, tile_rows)
    block = rng.standard_normal((rows, wl.dim), dtype=np.float32) * np.float32(0.01)
    if rows == wl.vocab:
        return block
    out = np.empty((wl.vocab, wl.dim), dtype=np.float32)
    for lo in range(0, wl.vocab, rows):
        hi = min(lo + rows, wl.vocab)
        out[lo:hi] = block[: hi - lo]
    return out
