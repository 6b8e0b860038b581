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


# ------------------------------------------------------------------------------------------
# the (1 + eps) rule of Sec. 4.5
# ------------------------------------------------------------------------------------------
def _eps_path_fixture(dtype):
    f = json.load(open(os.path.join(GOLD, "eps_path.json")))
    xs = f["xs"]
    n = len(xs)
    pts = np.zeros((n, 4), dtype)
    pts[:, 0] = xs
    g = np.full((n, 2), NONE, np.uint32)
    for i in range(n):
        nb = [j for j in (i - 1, i + 1) if 0 <= j < n]
        g[i, :len(nb)] = nb
    q = np.zeros(4, dtype)
    q[0] = f["query_x"]
    return f, pts, g, q


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_eps_rule_hand_worked_path(oracle, dtype):
    f, pts, g, q = _eps_path_fixture(dtype)
    ds = oracle.Dataset(pts, 0)
    for c in f["cases"]:
        st = oracle.Stats()
        v_ids, v_d, k_ids, k_d = oracle.greedy_search(ds, g, f["start"], q, f["L"], c["k"], stats=st, eps=c["eps"])
        assert v_ids.tolist() == c["expect_V"], c
        assert v_d.tolist() == [f["dists"][i] for i in c["expect_V"]]
        assert k_ids.tolist() == c["expect_K"], c
        assert st.evals == f["expect_evals"]


@pytest.mark.parametrize("dtype,metric", [(np.uint8, 0), (np.int8, 0), (np.float32, 0), (np.float32, 1)])
def test_eps_rule_cuts_a_prefix_and_keeps_the_k_nearest_of_it(oracle, dtype, metric):
    """Whatever eps, the search is the unrestricted one cut short: its visited sequence is a
    prefix of the unrestricted sequence, growing with eps; a huge eps changes nothing; the k
    results are the k nearest of what was visited; and where it stopped early, the next vertex
    in line was indeed beyond the bound (checked from the visited sets alone, in numpy)."""
    rng = np.random.default_rng(21)
    n, d, R, L, k = 300, 6, 6, 12, 4
    pts = _rand_points(rng, n, d, dtype)
    if metric == 1:
        pts /= np.linalg.norm(pts, axis=1, keepdims=True)
    ds = oracle.Dataset(pts, metric)
    g = _random_graph(rng, n, R)
    shorter = 0
    for _ in range(40):
        q = _rand_points(rng, 1, d, dtype)[0]
        s = int(rng.integers(n))
        v_off, _, k_off, _ = oracle.greedy_search(ds, g, s, q, L, k)
        prev = 0
        for eps in (0.0, 0.05, 0.25, 1.0, 16000.0):
            v, vd, kk, kd = oracle.greedy_search(ds, g, s, q, L, k, eps=eps)
            assert v.tolist() == v_off[:len(v)].tolist()
            assert len(v) >= prev
            prev = len(v)
            if eps == 16000.0:
                assert len(v) == len(v_off) and kk.tolist() == k_off.tolist()
            ek, ed = exact_knn(pts, q, k, metric, subset=v.tolist())
            m = min(k, len(v))
            assert kk[:m].tolist() == ek[:m].tolist()
            if len(v) < len(v_off):
                shorter += 1
                # At an early stop the beam's first k entries are all visited (an unvisited one
                # would be within the bound), so the k-th nearest visited vertex IS d_k, and the
                # vertex the unrestricted search expands next must lie beyond its bound.
                assert len(v) >= k
                nxt = int(v_off[len(v)])
                dn = np_dists_to(pts[nxt:nxt + 1], q, metric)[0]
                dk = ed[k - 1]
                if dtype == np.float32:
                    bound = np.float32(dk) + np.float32(eps) * np.abs(np.float32(dk))
                    assert np.float32(dn) > bound
                else:
                    assert int(dn) * 65536 > int(dk) * (65536 + int(round(eps * 65536)))
    assert shorter > 20
