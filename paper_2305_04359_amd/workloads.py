"""Seeded synthetic workloads with the shapes, dtypes and metrics of the paper's data sets.

This module only draws inputs.  It holds none of the method's arithmetic and is the one piece
shared by the HIP path's tests, the CPU oracle's tests and the benchmark: both sides receive the
very same arrays.  The data sets named in Sec. 5 of the paper (128-d uint8 SIFT descriptors,
100-d int8 vectors, 200-d float vectors searched by inner product with out-of-distribution
queries) are not available offline; these generators stand in for them.

Rows are produced in blocks of ``BLOCK`` rows, block ``b`` of a stream seeded by
``(seed, stream, b)``, so any block can be regenerated on its own.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BLOCK = 65536
DATA_SEED = 2305
QUERY_SEED = 4359
BUILD_SEED = 1

L2SQ, MIPS = 0, 1


def _rng(seed: int, stream: int, block: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, block])))


def _blocks(n: int):
    for b, lo in enumerate(range(0, n, BLOCK)):
        yield b, lo, min(n, lo + BLOCK)


def gaussian_mixture_u8(n, d, centers, sigma, seed, stream, lo=0, hi=255, dtype=np.uint8):
    """Rows = clip(round(center[k] + sigma * g), lo, hi), k uniform over the centres.
    Blocks are independent streams, so large inputs are drawn by a few threads at once; the
    result does not depend on how many."""
    out = np.empty((n, d), dtype)

    def draw(item):
        b, s, e = item
        g = _rng(seed, stream, b)
        k = g.integers(0, centers.shape[0], size=e - s)
        x = centers[k] + sigma * g.standard_normal((e - s, d), dtype=np.float32)
        out[s:e] = np.clip(np.rint(x), lo, hi).astype(dtype)

    items = list(_blocks(n))
    workers = min(16, os.cpu_count() or 1, len(items))
    if workers <= 1 or n < 4 * BLOCK:
        for it in items:
            draw(it)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(draw, items))
    return out


def centers_uniform(ncent, d, lo, hi, seed):
    return _rng(seed, 100, 0).uniform(lo, hi, size=(ncent, d)).astype(np.float32)


def centers_sift_like(ncent, d, seed):
    """Histogram-shaped centre coordinates: 40 * Exp(1) - 16, about a third of them negative,
    so that after adding noise and clipping at zero roughly 30 % of all entries are exact zeros."""
    e = _rng(seed, 101, 0).exponential(1.0, size=(ncent, d)).astype(np.float32)
    return 40.0 * e - 16.0


def centers_normal(ncent, d, scale, seed):
    return (scale * _rng(seed, 102, 0).standard_normal((ncent, d))).astype(np.float32)


def centers_sphere(ncent, d, seed):
    c = _rng(seed, 103, 0).standard_normal((ncent, d))
    return (c / np.linalg.norm(c, axis=1, keepdims=True)).astype(np.float32)


def sphere_mixture_f32(n, centers, sigma, seed, stream):
    d = centers.shape[1]
    out = np.empty((n, d), np.float32)
    for b, s, e in _blocks(n):
        g = _rng(seed, stream, b)
        k = g.integers(0, centers.shape[0], size=e - s)
        x = centers[k].astype(np.float64) + sigma * g.standard_normal((e - s, d))
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        out[s:e] = x.astype(np.float32)
    return out


def rotation_by_angle(d, degrees, seed):
    """An orthogonal matrix that turns every vector by exactly `degrees`: the same plane
    rotation in d/2 orthogonal planes of a random basis."""
    assert d % 2 == 0
    q, _ = np.linalg.qr(_rng(seed, 104, 0).standard_normal((d, d)))
    t = np.deg2rad(degrees)
    blk = np.zeros((d, d))
    c, s = np.cos(t), np.sin(t)
    for i in range(0, d, 2):
        blk[i, i], blk[i, i + 1], blk[i + 1, i], blk[i + 1, i + 1] = c, -s, s, c
    return q @ blk @ q.T


@dataclass
class Workload:
    name: str
    points: np.ndarray
    queries: np.ndarray
    metric: int
    R: int
    L: int
    alpha: float
    k: int = 10
    search_L: tuple = ()
    seed: int = BUILD_SEED
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n(self):
        return self.points.shape[0]

    @property
    def d(self):
        return self.points.shape[1]

    @property
    def theta(self):
        return max(1, self.n // 50)


def c1(n=10_000, nq=1_000):
    """n x 128 uint8 from 32 isotropic Gaussians, centres uniform in [32,224], sigma 20."""
    cen = centers_uniform(32, 128, 32.0, 224.0, DATA_SEED)
    return Workload("C1", gaussian_mixture_u8(n, 128, cen, 20.0, DATA_SEED, 0),
                    gaussian_mixture_u8(nq, 128, cen, 20.0, QUERY_SEED, 1), L2SQ,
                    R=32, L=64, alpha=1.2, search_L=(20, 30, 40, 50, 60, 80),
                    note="stand-in for a small SIFT-like set")


def c2(n=1_000_000, nq=10_000):
    """n x 128 uint8, SIFT-like: 1,024 clusters, non-negative, about 30 % zeros."""
    cen = centers_sift_like(1024, 128, DATA_SEED)
    return Workload("C2", gaussian_mixture_u8(n, 128, cen, 12.0, DATA_SEED, 0),
                    gaussian_mixture_u8(nq, 128, cen, 12.0, QUERY_SEED, 1), L2SQ,
                    R=64, L=128, alpha=1.2,
                    search_L=(10, 11, 12, 13, 14, 15, 16, 18, 20, 30, 40, 50, 60, 80, 100, 120, 150, 200),
                    note="stand-in for BIGANN-1M (128-d uint8, L2)")


def c3(n=1_000_000, nq=10_000):
    """n x 100 int8 from 1,024 Gaussians, sigma 25, clipped to [-127,127]."""
    cen = centers_normal(1024, 100, 40.0, DATA_SEED)
    return Workload("C3",
                    gaussian_mixture_u8(n, 100, cen, 25.0, DATA_SEED, 0, -127, 127, np.int8),
                    gaussian_mixture_u8(nq, 100, cen, 25.0, QUERY_SEED, 1, -127, 127, np.int8),
                    L2SQ, R=64, L=128, alpha=1.2, search_L=(10, 15, 20, 25, 30, 35, 40, 50, 60, 80, 120, 200),
                    note="stand-in for MSSPACEV-1M (100-d int8, L2)")


def c4(n=1_000_000, nq=10_000):
    """n x 200 float32 unit vectors from 512 clusters on the sphere, inner-product search,
    queries from the same clusters turned by 30 degrees (out of distribution)."""
    cen = centers_sphere(512, 200, DATA_SEED)
    rot = rotation_by_angle(200, 30.0, DATA_SEED)
    qcen = (cen.astype(np.float64) @ rot.T).astype(np.float32)
    return Workload("C4", sphere_mixture_f32(n, cen, 0.05, DATA_SEED, 0),
                    sphere_mixture_f32(nq, qcen, 0.05, QUERY_SEED, 1), MIPS,
                    R=64, L=128, alpha=1.0, search_L=(10, 20, 30, 40, 45, 50, 60, 70, 80, 100, 120, 200),
                    note="stand-in for TEXT2IMAGE-1M (200-d float, inner product, OOD queries)")


def c5(n=100_000_000, nq=10_000):
    """C2's generator at 10^8 points."""
    w = c2(n, nq)
    w.name = "C5"
    w.note = "stand-in for BIGANN-100M"
    w.search_L = w.search_L + (250, 300, 400, 512, 700, 1000, 1400, 2048)
    return w


CONFIGS = {"C1": c1, "C2": c2, "C3": c3, "C4": c4, "C5": c5}


def make(name: str, n: int | None = None, nq: int | None = None) -> Workload:
    f = CONFIGS[name]
    kw = {}
    if n is not None:
        kw["n"] = n
    if nq is not None:
        kw["nq"] = nq
    return f(**kw)
