"""Pins for the oracle's schedule, insertion order, Alg. 2 and Alg. 3."""
import json
import os

import numpy as np
import pytest

from helpers import NONE, audit_prune, recall_at_k, row_list
from paper_2305_04359_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_schedule_closed_form(oracle):
    b = oracle.schedule(9999, 200).astype(np.int64)
    sizes = np.diff(b)
    assert b[0] == 0 and b[-1] == 9999
    assert sizes[:7].tolist() == [2, 4, 8, 16, 32, 64, 128]
    assert (sizes[7:-1] == 200).all() and 0 < sizes[-1] <= 200
    assert len(sizes) == 7 + -(-(9999 - 254) // 200) == 56
    # every batch is at most one larger than everything inserted before it (start vertex
    # included), and never above theta
    for theta in (1, 3, 50, 10 ** 6):
        b = oracle.schedule(1000, theta).astype(np.int64)
        sizes = np.diff(b)
        assert (sizes >= 1).all() and (sizes <= theta).all() and sizes.sum() == 1000
        assert all(sizes[i] <= b[i] + 2 for i in range(len(sizes)))
        grow = [i for i in range(len(sizes) - 1) if sizes[i] < theta]
        assert all(sizes[i] == b[i] + 2 for i in grow)
    assert oracle.schedule(0, 5).tolist() == [0]
    assert np.diff(oracle.schedule(5, 1).astype(np.int64)).tolist() == [1] * 5


def _splitmix64(state):
    state = (state + 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & (2 ** 64 - 1)
    return state, z ^ (z >> 31)


def test_insertion_order(oracle):
    # published SplitMix64 outputs for seed 0
    s, a = _splitmix64(0); s, b = _splitmix64(s); s, c = _splitmix64(s)
    assert (a, b, c) == (0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F)
    for n, start, seed in [(10, 3, 0), (1000, 0, 1), (1000, 999, 12345678901234567)]:
        got = oracle.insertion_order(n, start, seed)
        ids = [i for i in range(n) if i != start]
        st = seed
        for i in range(len(ids) - 1, 0, -1):
            st, r = _splitmix64(st)
            j = (r * (i + 1)) >> 64
            ids[i], ids[j] = ids[j], ids[i]
        assert got.tolist() == ids
        assert sorted(got.tolist()) == [i for i in range(n) if i != start]
    assert oracle.insertion_order(1000, 0, 1).tolist() != oracle.insertion_order(1000, 0, 2).tolist()


def test_start_vertex(oracle):
    rng = np.random.default_rng(0)
    for dtype in (np.uint8, np.int8, np.float32):
        if dtype == np.float32:
            pts = rng.standard_normal((500, 12)).astype(np.float32)
        else:
            pts = rng.integers(0 if dtype == np.uint8 else -127, 128, (500, 12)).astype(dtype)
        pts[400] = pts[77]
        ds = oracle.Dataset(pts, 0)
        x = pts.astype(np.float64)
        sc = ((x - x.mean(0)) ** 2).sum(1)
        s = oracle.start_vertex(ds)
        assert sc[s] <= sc.min() * (1 + 1e-12) + 1e-9
        if dtype != np.float32:
            # exact integer score and smallest id on ties
            X = pts.astype(object)
            S = X.sum(0)
            score = [500 * int((r * r).sum()) - 2 * int((r * S).sum()) for r in X]
            assert s == score.index(min(score))
    # a tie between identical points goes to the smaller id
    pts = np.zeros((4, 4), np.uint8); pts[0, 0] = 0; pts[3, 0] = 12; pts[1, 0] = 6; pts[2, 0] = 6
    assert oracle.start_vertex(oracle.Dataset(pts, 0)) == 1


def test_hand_worked_five_point_build(oracle):
    f = json.load(open(os.path.join(GOLD, "five_point_build.json")))
    pts = np.zeros((5, 4), np.int8)
    pts[:, 0] = f["xs"]
    ds = oracle.Dataset(pts, 0)
    order = np.array(f["order"], np.uint32)
    b = oracle.schedule(4, f["theta"]).astype(int)
    assert [order[b[i]:b[i + 1]].tolist() for i in range(len(b) - 1)] == f["expect_batches"]
    g1, _ = oracle.build(ds, f["R"], f["L"], f["alpha"], theta=f["theta"], start=f["start"],
                         order=order, max_rounds=1)
    assert [row_list(r) for r in g1] == f["expect_after_round_1"]
    for threads in (1, 3):
        g, s = oracle.build(ds, f["R"], f["L"], f["alpha"], theta=f["theta"], start=f["start"],
                            order=order, threads=threads)
        assert s == f["start"]
        assert [row_list(r) for r in g] == f["expect_graph"]


@pytest.fixture(scope="module")
def small():
    w = W.c1(n=1500, nq=200)
    return w


def test_batch_of_one_equals_sequential_insert(oracle, small):
    """theta = 1 makes every batch a single point; Alg. 3 must then coincide with running
    Alg. 2 point by point."""
    ds = oracle.Dataset(small.points[:400], 0)
    s = oracle.start_vertex(ds)
    order = oracle.insertion_order(400, s, 7)
    a, _ = oracle.build(ds, 8, 16, 1.2, theta=1, start=s, order=order)
    b = oracle.build_sequential(ds, 8, 16, 1.2, s, order)
    assert (a == b).all()
    # and a larger theta gives a different graph (the batches really see a stale snapshot)
    c, _ = oracle.build(ds, 8, 16, 1.2, theta=50, start=s, order=order)
    assert (a != c).any()


def test_round_by_round_invariants(oracle, small):
    """After every round: rows are compact, duplicate-free, loop-free and within R; points
    not yet inserted are untouched and unreferenced; the round's new points have no edge
    among themselves; every row written in the round is explained by the listing."""
    n = 600
    pts = small.points[:n]
    ds = oracle.Dataset(pts, 0)
    R, L, alpha, theta = 6, 12, 1.2, 40
    s = oracle.start_vertex(ds)
    order = oracle.insertion_order(n, s, 3)
    bounds = oracle.schedule(n - 1, theta).astype(int)
    prev = oracle.empty_graph(n, R)
    reprunes = 0
    for r in range(1, len(bounds)):
        g, _ = oracle.build(ds, R, L, alpha, theta=theta, start=s, order=order, max_rounds=r)
        batch = order[bounds[r - 1]:bounds[r]].tolist()
        inserted = set(order[:bounds[r]].tolist()) | {s}
        bset = set(batch)
        for i in range(n):
            row = g[i]
            lst = row_list(row)
            assert (row[:len(lst)] != NONE).all() and (row[len(lst):] == NONE).all()
            assert len(set(lst)) == len(lst) and i not in lst
            assert all(x in inserted for x in lst)
            if i not in inserted:
                assert lst == []
            if i in bset:
                assert not (set(lst) & bset)
        # step 1 rows: prune of the visited set of a search on the previous snapshot
        sources = {}
        for p in batch:
            v_ids, _, _, _ = oracle.greedy_search(ds, prev, s, pts[p], L, 1)
            audit_prune(pts, pts[p], p, v_ids, row_list(g[p]), R, alpha)
            for b in row_list(g[p]):
                sources.setdefault(b, []).append(p)
        # step 2 rows
        for i in range(n):
            if i in bset:
                continue
            old = row_list(prev[i])
            if i not in sources:
                assert row_list(g[i]) == old
                continue
            U = old + sources[i]
            if len(U) <= R:
                assert row_list(g[i]) == U
            else:
                reprunes += 1
                audit_prune(pts, pts[i], i, U, row_list(g[i]), R, alpha)
        prev = g
    assert reprunes > 50
    full, _ = oracle.build(ds, R, L, alpha, theta=theta, start=s, order=order)
    assert (full == prev).all()


def test_deterministic_and_thread_independent(oracle, small):
    ds = oracle.Dataset(small.points, 0)
    a, s = oracle.build(ds, 16, 32, 1.2, seed=5, threads=1)
    b, _ = oracle.build(ds, 16, 32, 1.2, seed=5, threads=4)
    c, _ = oracle.build(ds, 16, 32, 1.2, seed=5, threads=4)
    assert (a == b).all() and (b == c).all()
    d, _ = oracle.build(ds, 16, 32, 1.2, seed=6, threads=4)
    assert (a != d).any()


def test_quality(oracle, small):
    """The built graph answers queries well, recall grows with L, and the prefix-doubling
    build is about as good as the sequential one (Sec. 3.1, batch size truncation)."""
    ds = oracle.Dataset(small.points, 0)
    gt, _ = oracle.brute_force(ds, small.queries, 10)
    g, s = oracle.build(ds, 16, 32, 1.2, seed=1, threads=4)
    rec = []
    for L in (10, 20, 40, 80):
        ids, dists = oracle.search_batch(ds, g, s, small.queries, 10, L, threads=4)
        rec.append(recall_at_k(ids, gt))
        assert (np.diff(dists.astype(np.int64), axis=1) >= 0).all()
    assert rec == sorted(rec) and rec[-1] > 0.97
    order = oracle.insertion_order(ds.n, s, 1)
    gs = oracle.build_sequential(ds, 16, 32, 1.2, s, order)
    ids, _ = oracle.search_batch(ds, gs, s, small.queries, 10, 40, threads=4)
    ids_b, _ = oracle.search_batch(ds, g, s, small.queries, 10, 40, threads=4)
    assert abs(recall_at_k(ids, gt) - recall_at_k(ids_b, gt)) < 0.03
