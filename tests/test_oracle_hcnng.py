"""Pins for the oracle's clustering-based builder (ParlayHCNNG, Sec. 3.2 and 4.3)."""
import json
import os

import numpy as np
import pytest

from helpers import NONE, audit_prune, np_dist, recall_at_k, row_list
from paper_2305_04359_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")
M64 = 2 ** 64 - 1


def _stream(seed, k):
    """The (k+1)-th output of SplitMix64(seed), in Python integers."""
    z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _tree(points, Ls, seed, tree):
    """The cluster tree re-stated: returns the leaves (lists of ids) in left-to-right order."""
    leaves = []

    def split(ids, node, depth):
        c = len(ids)
        if c <= Ls:
            leaves.append(ids)
            return
        k = 2 * ((tree << 40) + node)
        i1 = (_stream(seed, k) * c) >> 64
        i2 = (_stream(seed, k + 1) * (c - 1)) >> 64
        if i2 >= i1:
            i2 += 1
        p1, p2 = points[ids[i1]], points[ids[i2]]
        left = [x for x in ids if np_dist(points[x], p1) <= np_dist(points[x], p2)] if depth < 39 else []
        right = [x for x in ids if np_dist(points[x], p1) > np_dist(points[x], p2)] if depth < 39 else []
        if not left or not right:
            left, right = ids[:(c + 1) // 2], ids[(c + 1) // 2:]
        split(left, 2 * node, depth + 1)
        split(right, 2 * node + 1, depth + 1)

    split(list(range(len(points))), 1, 0)
    return leaves


def _leaf(points, ids, s, l):
    """Edge-restricted, degree-bounded Kruskal re-stated."""
    c = len(ids)
    k = min(l, c - 1)
    pairs = set()
    for a in ids:
        near = sorted((np_dist(points[a], points[b]), b) for b in ids if b != a)[:k]
        for dist, b in near:
            pairs.add((dist, min(a, b), max(a, b)))
    comp = {x: x for x in ids}
    deg = {x: 0 for x in ids}

    def find(x):
        while comp[x] != x:
            x = comp[x]
        return x

    out = []
    for dist, u, v in sorted(pairs):
        if deg[u] >= s or deg[v] >= s or find(u) == find(v):
            continue
        comp[find(u)] = find(v)
        deg[u] += 1
        deg[v] += 1
        out.append([u, v])
    return out


@pytest.fixture(scope="module")
def small():
    return W.c1(n=2500, nq=200)


def test_cluster_tree(oracle, small):
    pts = small.points[:1200]
    ds = oracle.Dataset(pts, 0)
    for Ls, seed, tree in [(100, 1, 0), (100, 1, 7), (37, 99, 3), (1200, 5, 0), (2, 5, 1)]:
        perm, off = oracle.hcnng_tree(ds, Ls, seed, tree)
        leaves = [perm[off[j]:off[j + 1]].tolist() for j in range(len(off) - 1)]
        assert sorted(perm.tolist()) == list(range(1200))
        assert all(1 <= len(x) <= Ls and x == sorted(x) for x in leaves)
        assert leaves == _tree(pts, Ls, seed, tree)
    # different trees cut differently
    a, _ = oracle.hcnng_tree(ds, 100, 1, 0)
    b, _ = oracle.hcnng_tree(ds, 100, 1, 1)
    assert (a != b).any()
    # equal points cannot be separated: the order is cut in the middle, all the way down
    same = np.full((50, 8), 9, np.uint8)
    perm, off = oracle.hcnng_tree(oracle.Dataset(same, 0), 8, 1, 0)
    assert perm.tolist() == list(range(50)) and np.diff(off).tolist() == [7, 6, 6, 6, 7, 6, 6, 6]
    assert [len(x) for x in _tree(same, 8, 1, 0)] == [7, 6, 6, 6, 7, 6, 6, 6]


def test_leaf_worked_by_hand(oracle):
    g = json.load(open(os.path.join(GOLD, "hcnng_leaf.json")))
    pts = np.zeros((len(g["xs"]), g["d"]), np.uint8)
    pts[:, 0], pts[:, 1] = g["xs"], g["ys"]
    for dtype in (np.uint8, np.float32):
        ds = oracle.Dataset(pts.astype(dtype), 0)
        for c in g["cases"]:
            got = oracle.hcnng_leaf(ds, np.arange(len(pts)), c["s"], c["l"])
            assert got.tolist() == c["expect_pairs"], c


def test_leaf_against_scipy_and_restatement(oracle, small):
    from scipy.sparse.csgraph import minimum_spanning_tree
    pts = small.points
    ds = oracle.Dataset(pts, 0)
    rng = np.random.default_rng(3)
    for cnt in (2, 3, 17, 120):
        ids = np.sort(rng.choice(len(pts), cnt, replace=False)).astype(np.uint32)
        # neither bound restricts: a minimum spanning tree of the complete graph
        got = oracle.hcnng_leaf(ds, ids, cnt, cnt)
        assert len(got) == cnt - 1
        w = np.array([[np_dist(pts[a], pts[b]) for b in ids] for a in ids], dtype=np.float64)
        assert sum(np_dist(pts[u], pts[v]) for u, v in got) == int(minimum_spanning_tree(w).sum())
        # both bounds at work
        for s, l in ((3, 10), (2, 4), (1, 3), (3, 1)):
            got = oracle.hcnng_leaf(ds, ids, s, l)
            assert got.tolist() == _leaf(pts, ids.tolist(), s, l)
            deg = np.bincount(got.ravel(), minlength=len(pts)) if len(got) else np.zeros(1)
            assert deg.max() <= s
    assert oracle.hcnng_leaf(ds, np.array([5], np.uint32), 3, 10).shape == (0, 2)


def test_whole_build(oracle, small):
    n, T, Ls, s, l, R, alpha = 1500, 6, 120, 3, 10, 20, 1.2
    pts = small.points[:n]
    ds = oracle.Dataset(pts, 0)
    st = oracle.HcnngStats()
    g = oracle.hcnng_build(ds, T, Ls, s, l, R, alpha, seed=4, threads=0, stats=st)
    # the neighbour sets, from the re-stated pieces
    nb = [set() for _ in range(n)]
    nleaves = nedges = 0
    for t in range(T):
        for leaf in _tree(pts, Ls, 4, t):
            nleaves += 1
            for u, v in _leaf(pts, leaf, s, l) if len(leaf) > 1 else []:
                nb[u].add(v)
                nb[v].add(u)
                nedges += 1
    assert (st.leaves, st.tree_edges, st.neighbours) == (nleaves, nedges, sum(len(x) for x in nb))
    for p in range(0, n, 7):
        cand = np.array(sorted(nb[p]), np.uint32)
        assert row_list(g[p]) == oracle.prune(ds, pts[p], p, cand, R, alpha).tolist()
        audit_prune(pts, pts[p], p, cand, row_list(g[p]), R, alpha)
    assert all(set(row_list(g[p])) <= nb[p] for p in range(n))
    # same result whatever the thread count
    assert (oracle.hcnng_build(ds, T, Ls, s, l, R, alpha, seed=4, threads=1) == g).all()
    # the graph answers queries (the search is the flat graph's, from the point nearest the mean)
    gt, _ = oracle.brute_force(ds, small.queries, 10)
    ids, _ = oracle.search_batch(ds, g, oracle.start_vertex(ds), small.queries, 10, 40, threads=0)
    assert recall_at_k(ids, gt) > 0.9
