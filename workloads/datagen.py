"""Seeded synthetic float32 workloads.

This module only draws numbers: it holds none of the method's arithmetic
(no encoding, no code distance, no search) and is the one piece of code that
both the CPU oracle's tests and the GPU path's tests/benchmark use, so that both
sides see the same inputs.

The five workloads stand in for the datasets of the paper's Table 4 / Table 5
(which are not available offline): unit-norm, clustered, anisotropic vectors for
the contrastive-embedding shapes (384 / 768 / 3072-d, 1M vectors, 10k queries),
and unnormalised i.i.d. Gaussian vectors for the structureless regime.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n: int            # base vectors
    d: int            # dimension
    nq: int           # queries
    kind: str         # "tiny" | "powerlaw" | "gaussian"
    clusters: int     # 0 for "gaussian"
    R: int            # graph degree cap (2m in the paper)
    L: int            # construction beam width (ef_c in the paper)
    alpha: float      # diversity factor of the edge selection
    k: int
    efs: tuple        # ef values the workload is searched with
    metric: str       # ground-truth metric: "cosine" | "l2"
    seed_base: int
    seed_query: int


WORKLOADS = {
    # Tiny: 16 equally likely clusters, noise 0.3/sqrt(d)
    "C1": Workload("C1", 10_000, 128, 100, "tiny", 16, 32, 64, 1.2, 10, (64,), "cosine", 1001, 2001),
    # 768-d headline shape (the paper's Cohere-1M row of Table 5)
    "C2": Workload("C2", 1_000_000, 768, 10_000, "powerlaw", 1024, 64, 128, 1.2, 10, (16, 32, 64, 128), "cosine", 1002, 2002),
    # 384-d: short codes (96 B), gather-latency bound
    "C3": Workload("C3", 1_000_000, 384, 10_000, "powerlaw", 512, 64, 128, 1.2, 10, (64,), "cosine", 1003, 2003),
    # 3072-d: long codes (768 B)
    "C4": Workload("C4", 1_000_000, 3072, 10_000, "powerlaw", 2048, 64, 128, 1.2, 10, (64,), "cosine", 1004, 2004),
    # not one of the five contract workloads: low-rank data whose neighbours differ in direction (the regime
    # the paper calls compatible), used to show the path end to end at a recall that means something
    "H2": Workload("H2", 1_000_000, 768, 10_000, "lowrank", 32, 64, 128, 1.2, 10, (64,), "cosine", 1012, 2012),
    # not a contract workload either: the shape of the paper's scalability study (5M x 1024-d, Table 12) with the
    # low-rank law, so that recall at 1M (scaled(n=1_000_000) takes the first 1M rows) and at 5M can be compared
    "S5": Workload("S5", 5_000_000, 1024, 10_000, "lowrank", 32, 64, 128, 1.2, 10, (64, 128, 256, 512, 1024), "cosine",
                   1013, 2013),
    # structureless boundary case
    "C5": Workload("C5", 1_000_000, 512, 10_000, "gaussian", 0, 64, 128, 1.2, 10, (64,), "l2", 1005, 2005),
}


def scaled(name: str, n: int | None = None, nq: int | None = None, **kw) -> Workload:
    """A workload with the same generator and shape parameters but fewer vectors / queries."""
    w = WORKLOADS[name]
    return replace(w, n=n if n is not None else w.n, nq=nq if nq is not None else w.nq, **kw)


def _normalise_rows(x: np.ndarray) -> None:
    nrm = np.sqrt(np.einsum("ij,ij->i", x, x, dtype=np.float64))
    nrm[nrm == 0] = 1.0
    x /= nrm[:, None].astype(np.float32)


def _cluster_sizes(n: int, clusters: int, exponent: float) -> np.ndarray:
    """Sizes proportional to (c+1)^-exponent, at least one each, summing to n (largest remainder)."""
    w = (np.arange(clusters, dtype=np.float64) + 1.0) ** (-exponent)
    w /= w.sum()
    free = n - clusters
    assert free >= 0, "need at least one vector per cluster"
    quota = w * free
    base = np.floor(quota).astype(np.int64)
    rem = free - int(base.sum())
    order = np.argsort(-(quota - base), kind="stable")
    base[order[:rem]] += 1
    sizes = base + 1
    assert sizes.sum() == n
    return sizes


class _Model:
    """Cluster centres and noise law of one workload (drawn once from the base seed)."""

    def __init__(self, w: Workload):
        self.w = w
        rng = np.random.Generator(np.random.PCG64(w.seed_base))
        if w.kind == "gaussian":
            return
        if w.kind == "lowrank":
            # x = normalise(z A + small noise): z standard normal in `clusters` latent dimensions
            self.basis = rng.standard_normal((w.clusters, w.d), dtype=np.float32) / np.float32(np.sqrt(w.clusters))
            return
        c = rng.standard_normal((w.clusters, w.d), dtype=np.float32)
        _normalise_rows(c)
        self.centres = c
        if w.kind == "tiny":
            self.scale = np.full(w.d, 0.3 / np.sqrt(w.d), dtype=np.float32)
            self.prob = np.full(w.clusters, 1.0 / w.clusters)
        else:
            u = rng.uniform(np.log(0.5), np.log(2.0), size=w.d)
            self.scale = ((0.25 / np.sqrt(w.d)) * np.exp(u)).astype(np.float32)
            # queries pick a cluster with probability proportional to its size
            self.prob = _cluster_sizes(w.n, w.clusters, 1.5) / float(w.n)

    def draw(self, labels: np.ndarray, seed: list) -> np.ndarray:
        w = self.w
        out = np.empty((labels.shape[0], w.d), dtype=np.float32)

        def fill_lowrank(c, s, e):
            rng = _chunk_rng(seed, c)
            z = rng.standard_normal((e - s, w.clusters), dtype=np.float32)
            g = z @ self.basis
            g += np.float32(0.05) * rng.standard_normal((e - s, w.d), dtype=np.float32)
            _normalise_rows(g)
            out[s:e] = g

        if w.kind == "lowrank":
            _for_chunks(labels.shape[0], fill_lowrank)
            return out

        def fill(c, s, e):
            g = _chunk_rng(seed, c).standard_normal((e - s, w.d), dtype=np.float32)
            g *= self.scale[None, :]
            g += self.centres[labels[s:e]]
            _normalise_rows(g)
            out[s:e] = g

        _for_chunks(labels.shape[0], fill)
        return out


CHUNK = 32768
THREADS = min(16, os.cpu_count() or 1)


def _chunk_rng(seed: list, c: int) -> np.random.Generator:
    """Every chunk of rows has a generator of its own, so chunks can be drawn in any order."""
    return np.random.Generator(np.random.PCG64(list(seed) + [c]))


def _for_chunks(n: int, fn) -> None:
    spans = [(c, s, min(n, s + CHUNK)) for c, s in enumerate(range(0, n, CHUNK))]
    if len(spans) <= 1 or THREADS <= 1:
        for sp in spans:
            fn(*sp)
        return
    with ThreadPoolExecutor(THREADS) as ex:
        list(ex.map(lambda sp: fn(*sp), spans))


def make_base(w: Workload) -> np.ndarray:
    """Base vectors [n, d] float32."""
    m = _Model(w)
    rng = np.random.Generator(np.random.PCG64([w.seed_base, 1]))
    if w.kind == "gaussian":
        out = np.empty((w.n, w.d), dtype=np.float32)

        def fill(c, s, e):
            out[s:e] = _chunk_rng([w.seed_base, 3], c).standard_normal((e - s, w.d), dtype=np.float32)

        _for_chunks(w.n, fill)
        return out
    if w.kind == "lowrank":
        return m.draw(np.zeros(w.n, dtype=np.int64), [w.seed_base, 3])
    if w.kind == "tiny":
        labels = rng.integers(0, w.clusters, size=w.n)
    else:
        sizes = _cluster_sizes(w.n, w.clusters, 1.5)
        labels = np.repeat(np.arange(w.clusters), sizes)
        labels = labels[rng.permutation(w.n)]  # ids carry no cluster locality
    return m.draw(labels, [w.seed_base, 3])


def make_queries(w: Workload) -> np.ndarray:
    """Queries [nq, d] float32 from the same law as the base vectors (fresh noise)."""
    m = _Model(w)
    rng = np.random.Generator(np.random.PCG64([w.seed_query, 2]))
    if w.kind == "gaussian":
        return _chunk_rng([w.seed_query, 4], 0).standard_normal((w.nq, w.d), dtype=np.float32)
    if w.kind == "lowrank":
        return m.draw(np.zeros(w.nq, dtype=np.int64), [w.seed_query, 4])
    labels = rng.choice(w.clusters, size=w.nq, p=m.prob)
    return m.draw(labels, [w.seed_query, 4])


def random_regular_graph(n: int, R: int, seed: int, fill: float = 1.0) -> np.ndarray:
    """A random directed graph [n, R] uint32 (no self loops; empty slots = 0xFFFFFFFF).

    Not a navigable index: used where a test only needs *some* adjacency of the right shape.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    adj = rng.integers(0, n - 1, size=(n, R), dtype=np.int64)
    adj += adj >= np.arange(n)[:, None]  # skip self
    adj = adj.astype(np.uint32)
    if fill < 1.0:
        adj[rng.random((n, R)) > fill] = 0xFFFFFFFF
    return adj
