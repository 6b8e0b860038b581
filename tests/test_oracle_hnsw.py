"""Pins for the oracle's layered index (ParlayHNSW, Sec. 4.2)."""
import json
import os

import numpy as np
import pytest

from helpers import NONE, recall_at_k, row_list
from paper_2305_04359_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")
M64 = 2 ** 64 - 1


def _level(seed, i, m):
    """The level rule in Python integers: r = the (i+1)-th SplitMix64 output for `seed`."""
    z = (seed + (i + 1) * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    r = z ^ (z >> 31)
    l = 0
    while M64 // m ** (l + 1) > 0 and r <= M64 // m ** (l + 1):
        l += 1
    return l


@pytest.fixture(scope="module")
def small():
    return W.c1(n=3000, nq=200)


def test_levels(oracle):
    # by hand from the published first outputs of SplitMix64 for seed 0, m = 2 (thresholds
    # 0x7FFF.., 0x3FFF.., 0x1FFF.., ...): 0xE220A8397B1DCDAF is above the first, 0x6E789E6AA1B965F4
    # passes one, 0x06C45D188009454F passes five (0x07FF.. but not 0x03FF..)
    assert [oracle.hnsw_level(0, i, 2) for i in range(3)] == [0, 1, 5]
    for seed, m in [(0, 2), (1, 32), (99, 5), (12345678901234567, 16)]:
        assert [oracle.hnsw_level(seed, i, m) for i in range(3000)] == [_level(seed, i, m) for i in range(3000)]
    # geometric law: P(level >= j) = m^-j
    n, m = 200_000, 4
    lev = np.array([oracle.hnsw_level(7, i, m) for i in range(n)])
    for j in range(1, 6):
        p = m ** -j
        assert abs((lev >= j).sum() - n * p) < 5 * np.sqrt(n * p * (1 - p)) + 1
    assert lev.max() <= 12


def test_every_level_zero_is_the_flat_build(oracle, small):
    """With one layer the index is the graph of Alg. 3 with R = 2m, the entry point (smallest id,
    all levels being equal) as start vertex."""
    n, m, efc = 800, 6, 24
    ds = oracle.Dataset(small.points[:n], 0)
    h = oracle.hnsw_build(ds, m, efc, 1.2, seed=3, theta=40, level=np.zeros(n, np.uint32))
    assert h.top == 0 and h.entry == 0
    flat, _ = oracle.build(ds, 2 * m, efc, 1.2, seed=3, theta=40, start=0)
    assert (h.layers[0] == flat).all()
    ids, dists, ent = oracle.hnsw_search_batch(ds, h, small.queries, 5, 20)
    fi, fd = oracle.search_batch(ds, flat, 0, small.queries, 5, 20)
    assert (ids == fi).all() and (dists == fd).all() and (ent == 0).all()


def test_batches_of_one_are_alg2_layer_by_layer(oracle, small):
    """theta = 1: every point walks down from the entry point (beam 1 above its level) and is
    inserted with Alg. 2 on each of its layers, the closest visited vertex leading one layer
    down.  Re-stated here with the single-point primitives."""
    n, m, efc = 500, 4, 12
    ds = oracle.Dataset(small.points[:n], 0)
    h = oracle.hnsw_build(ds, m, efc, 1.1, seed=11, theta=1)
    lev = np.array([_level(11, i, m) for i in range(n)])
    assert (h.level == lev).all() and h.top == lev.max() >= 2
    entry = int(np.flatnonzero(lev == lev.max())[0])
    assert h.entry == entry
    order = oracle.insertion_order(n, entry, 11)
    layers = [oracle.empty_graph(n, 2 * m if l == 0 else m) for l in range(h.top + 1)]
    for p in order:
        cur = entry
        for l in range(h.top, -1, -1):
            beam = 1 if lev[p] < l else efc
            _, _, k_ids, _ = oracle.greedy_search(ds, layers[l], cur, ds.points[p], beam, 1)
            if lev[p] >= l:
                oracle.insert(ds, layers[l], cur, int(p), efc, 1.1)
            cur = int(k_ids[0])
    for l in range(h.top + 1):
        assert (h.layers[l] == layers[l]).all(), f"layer {l}"


def test_layer_invariants_and_snapshot(oracle, small):
    n, m, efc = 3000, 8, 32
    ds = oracle.Dataset(small.points, 0)
    h = oracle.hnsw_build(ds, m, efc, 1.2, seed=1, threads=0)
    lev = h.level.astype(np.int64)
    assert h.top == lev.max() and lev[h.entry] == h.top
    for l, rows in enumerate(h.layers):
        members = np.flatnonzero(lev >= l)
        assert (rows[lev < l] == NONE).all()
        for v in members:
            row = row_list(rows[v])
            assert len(row) == len(set(row)) and v not in row
            assert all(lev[u] >= l for u in row)
            assert (rows[v][len(row):] == NONE).all()
            if v != h.entry and len(members) > 1:
                assert len(row) >= 1
    # deterministic, and independent of the thread count
    h2 = oracle.hnsw_build(ds, m, efc, 1.2, seed=1, threads=1)
    assert all((a == b).all() for a, b in zip(h.layers, h2.layers))
    # after any round: the round's points have no edges among themselves on any layer (they all
    # searched the layers as they stood before the round), later points are absent
    b = oracle.schedule(n - 1, n // 50).astype(np.int64)
    order = oracle.insertion_order(n, h.entry, 1)
    for r in (5, 9, 20):
        part = oracle.hnsw_build(ds, m, efc, 1.2, seed=1, max_rounds=r)
        batch = set(order[b[r - 1]:b[r]].tolist())
        later = order[b[r]:]
        for l, rows in enumerate(part.layers):
            assert (rows[later] == NONE).all() and not np.isin(rows, later).any()
            for v in batch:
                assert not (set(row_list(rows[v])) & batch)


def test_search_worked_by_hand(oracle):
    g = json.load(open(os.path.join(GOLD, "hnsw_descent.json")))
    xs, m = g["xs"], g["m"]
    n = len(xs)
    pts = np.zeros((n, g["d"]), np.uint8)
    pts[:, 0] = xs
    layers = []
    for l in range(len(g["layers"])):
        rows = oracle.empty_graph(n, 2 * m if l == 0 else m)
        for v, nb in g["layers"][str(l)].items():
            rows[int(v), :len(nb)] = nb
        layers.append(rows)
    h = oracle.Hnsw(m, np.array(g["level"], np.uint32), layers, g["entry"])
    for dtype in (np.uint8, np.float32):
        ds = oracle.Dataset(pts.astype(dtype), 0)
        for c in g["cases"]:
            q = np.zeros((1, g["d"]), dtype)
            q[0, 0] = c["query_x"]
            ids, dists, ent = oracle.hnsw_search_batch(ds, h, q, g["k"], g["L"])
            assert ent.tolist() == [c["expect_entry0"]]
            assert ids[0].tolist() == c["expect_ids"] and dists[0].tolist() == c["expect_dists"]


def test_quality(oracle, small):
    ds = oracle.Dataset(small.points, 0)
    h = oracle.hnsw_build(ds, 16, 64, 1.0, seed=1, threads=0)
    gt, _ = oracle.brute_force(ds, small.queries, 10)
    ids, _, _ = oracle.hnsw_search_batch(ds, h, small.queries, 10, 40, threads=0)
    assert recall_at_k(ids, gt) > 0.95
    flat, s = oracle.build(ds, 32, 64, 1.0, seed=1, threads=0)
    fi, _ = oracle.search_batch(ds, flat, s, small.queries, 10, 40, threads=0)
    assert abs(recall_at_k(ids, gt) - recall_at_k(fi, gt)) < 0.03
    # the (1 + eps) rule applies on the bottom layer only: eps = 0 with k = 1 stops at the first
    # vertex that is not the nearest so far, and can only lose recall
    ids0, _, ent = oracle.hnsw_search_batch(ds, h, small.queries, 10, 40, eps=0.0)
    assert recall_at_k(ids0, gt) <= recall_at_k(ids, gt)
    ids_big, _, ent2 = oracle.hnsw_search_batch(ds, h, small.queries, 10, 40, eps=1000.0)
    assert (ids_big == ids).all() and (ent == ent2).all()


def test_streaming_into_the_layered_index_continues_the_build(oracle, small):
    """An index over all points, its build cut at a batch boundary, is the index over the points
    before the cut with the rest streamed in (same levels, order and theta; ids in insertion
    order so that a prefix of the order is a prefix of the ids)."""
    n, m, efc, theta = 900, 5, 16, 60
    pts = small.points[:n]
    rng = np.random.default_rng(2)
    level = np.minimum(rng.geometric(0.6, n) - 1, 3).astype(np.uint32)
    level[0] = 3  # the entry point comes first
    order = np.arange(1, n, dtype=np.uint32)
    full = oracle.Dataset(pts, 0)
    whole = oracle.hnsw_build(full, m, efc, 1.2, theta=theta, level=level, order=order)
    assert whole.entry == 0 and whole.top == 3
    b = oracle.schedule(n - 1, theta).astype(np.int64)
    for r in (4, 9):
        n_old = int(b[r]) + 1
        head = oracle.hnsw_build(oracle.Dataset(pts[:n_old], 0), m, efc, 1.2, theta=theta, level=level[:n_old],
                                 order=order[:n_old - 1])
        grown = oracle.hnsw_insert_points(full, head, efc, 1.2, theta=theta, order=order[n_old - 1:],
                                          level=level[n_old:])
        assert (grown.level == whole.level).all()
        for l in range(whole.top + 1):
            assert (grown.layers[l] == whole.layers[l]).all(), f"cut {r}, layer {l}"
    # levels by the rule are capped at the index's highest layer
    head = oracle.hnsw_build(oracle.Dataset(pts[:300], 0), 2, efc, 1.2, seed=4)
    grown = oracle.hnsw_insert_points(full, head, efc, 1.2, seed=9, level_seed=4)
    want = np.array([min(_level(4, i, 2), head.top) for i in range(300, n)])
    assert (grown.level[300:] == want).all() and (grown.level[:300] == head.level).all()
    for l, rows in enumerate(grown.layers):
        assert (rows[grown.level < l] == NONE).all()
        assert all(len(row_list(rows[v])) >= 1 for v in np.flatnonzero(grown.level >= l) if v != grown.entry)
