"""Pins for the oracle's greedySearch (Alg. 1)."""
import json
import os
from collections import deque

import numpy as np
import pytest

from helpers import NONE, exact_knn, np_dists_to

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand_points(rng, n, d, dtype):
    if dtype == np.uint8:
        return rng.integers(0, 256, (n, d)).astype(np.uint8)
    if dtype == np.int8:
        return rng.integers(-127, 128, (n, d)).astype(np.int8)
    return rng.standard_normal((n, d)).astype(np.float32)


def _complete_graph(n):
    g = np.empty((n, n - 1), np.uint32)
    for i in range(n):
        g[i] = [j for j in range(n) if j != i]
    return g


def _random_graph(rng, n, R):
    g = np.full((n, R), NONE, np.uint32)
    for i in range(n):
        deg = rng.integers(0, R + 1)
        nb = rng.choice([j for j in range(n) if j != i], size=min(deg, n - 1), replace=False)
        g[i, :len(nb)] = nb
    return g


def _reachable(g, s):
    seen = {s}
    dq = deque([s])
    while dq:
        u = dq.popleft()
        for v in g[u]:
            v = int(v)
            if v != NONE and v not in seen:
                seen.add(v)
                dq.append(v)
    return seen


@pytest.mark.parametrize("dtype,metric", [(np.uint8, 0), (np.int8, 0), (np.float32, 0), (np.float32, 1)])
def test_complete_graph_gives_exact_knn(oracle, dtype, metric):
    """On a complete graph the first hop puts every vertex in the beam, which keeps the L
    closest: the result must be the exact k nearest neighbours."""
    rng = np.random.default_rng(11)
    n, d = 40, 8
    pts = _rand_points(rng, n, d, dtype)
    pts[7] = pts[3]  # an exact duplicate: ties must go to the smaller id
    ds = oracle.Dataset(pts, metric)
    g = _complete_graph(n)
    for trial in range(10):
        q = _rand_points(rng, 1, d, dtype)[0]
        for (L, k) in [(5, 5), (10, 3), (39, 10), (64, 40)]:
            for start in (0, int(rng.integers(n))):
                _, _, k_ids, k_d = oracle.greedy_search(ds, g, start, q, L, k)
                e_ids, e_d = exact_knn(pts, q, k, metric)
                assert k_ids.tolist() == e_ids.tolist()
                assert k_d.tolist() == e_d.tolist()


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_wide_beam_visits_the_reachable_set(oracle, dtype):
    """With L >= n nothing is ever cut, so V is the set reachable from s and K the exact
    nearest neighbours among it."""
    rng = np.random.default_rng(5)
    n, d, R = 60, 6, 3
    pts = _rand_points(rng, n, d, dtype)
    ds = oracle.Dataset(pts, 0)
    for trial in range(10):
        g = _random_graph(rng, n, R)
        s = int(rng.integers(n))
        q = _rand_points(rng, 1, d, dtype)[0]
        st = oracle.Stats()
        v_ids, v_d, k_ids, k_d = oracle.greedy_search(ds, g, s, q, n, 5, stats=st)
        reach = _reachable(g, s)
        assert set(v_ids.tolist()) == reach and len(v_ids) == len(reach)
        assert st.evals == len(reach) and st.hops == len(reach)
        e_ids, e_d = exact_knn(pts, q, min(5, len(reach)), 0, subset=reach)
        assert k_ids[:len(e_ids)].tolist() == e_ids.tolist()
        assert all(int(x) == NONE for x in k_ids[len(e_ids):])
        assert all(np.isinf(x) for x in k_d[len(e_ids):])
        # each V entry carries its own distance
        dd = np_dists_to(pts[v_ids], q)
        assert v_d.tolist() == dd.tolist()
        # V is in processing order: with nothing cut, each processed vertex was the
        # closest one discovered so far and not yet processed
        assert v_ids[0] == s


def test_hand_worked_path(oracle):
    f = json.load(open(os.path.join(GOLD, "path_search.json")))
    xs = f["xs"]
    n = len(xs)
    pts = np.zeros((n, 4), np.uint8)
    pts[:, 0] = xs
    g = np.full((n, 2), NONE, np.uint32)
    for i in range(n - 1):
        g[i, 0] = i + 1
    q = np.zeros(4, np.uint8)
    q[0] = f["query_x"]
    ds = oracle.Dataset(pts, 0)
    st = oracle.Stats()
    v_ids, v_d, k_ids, k_d = oracle.greedy_search(ds, g, f["start"], q, f["L"], f["k"], stats=st)
    assert v_ids.tolist() == f["expect_V"]
    assert v_d.tolist() == f["expect_V_dists"]
    assert k_ids.tolist() == f["expect_K"]
    assert k_d.tolist() == f["expect_K_dists"]
    assert st.evals == f["expect_evals"] and st.hops == len(f["expect_V"])


def test_beam_one_is_greedy_descent(oracle):
    """L = 1: the walk moves to the best neighbour while it improves, then stops."""
    rng = np.random.default_rng(3)
    n, d, R = 50, 4, 4
    pts = _rand_points(rng, n, d, np.uint8)
    ds = oracle.Dataset(pts, 0)
    for _ in range(20):
        g = _random_graph(rng, n, R)
        s = int(rng.integers(n)); q = _rand_points(rng, 1, d, np.uint8)[0]
        v_ids, _, k_ids, _ = oracle.greedy_search(ds, g, s, q, 1, 1)
        dist = np_dists_to(pts, q)
        cur = s; walk = [s]
        while True:
            nb = [int(x) for x in g[cur] if int(x) != NONE]
            best = min([(dist[x], x) for x in nb] + [(dist[cur], cur)])
            if best[1] == cur:
                break
            cur = best[1]; walk.append(cur)
        assert v_ids.tolist() == walk and int(k_ids[0]) == cur


def test_batch_and_bruteforce_agree_with_numpy(oracle):
    rng = np.random.default_rng(9)
    n, d = 300, 16
    pts = _rand_points(rng, n, d, np.int8)
    qs = _rand_points(rng, 20, d, np.int8)
    ds = oracle.Dataset(pts, 0)
    ids, dists = oracle.brute_force(ds, qs, 7, threads=2)
    for i in range(20):
        e_ids, e_d = exact_knn(pts, qs[i], 7)
        assert ids[i].tolist() == e_ids.tolist() and dists[i].tolist() == e_d.tolist()
    g = _complete_graph(n)
    ids2, d2 = oracle.search_batch(ds, g, 0, qs, 7, 9, threads=2)
    assert (ids2 == ids).all() and (d2 == dists).all()
    assert dists.dtype == np.int32
