"""GPU parity: the HIP path against the CPU oracle, element by element, through the C ABI.

Integer vectors (u8, i8): graphs, ids and distances must be identical.  f32: distances within
1e-5 relative (inner products: relative to sum |p_i q_i|), recall within 0.002.
"""
import json
import os

import numpy as np
import pytest

from helpers import NONE, dev, recall_at_k, row_list, say
from paper_2305_04359_amd import workloads as W

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def c1():
    return W.c1()


@pytest.fixture(scope="module")
def c1_oracle(oracle, c1):
    ds = oracle.Dataset(c1.points, 0)
    g, s = oracle.build(ds, c1.R, c1.L, c1.alpha, seed=c1.seed, threads=0)
    return ds, g, s


# ------------------------------------------------------------------------------------------
# a6 start vertex, a0 schedule / order
# ------------------------------------------------------------------------------------------
def test_start_vertex(env, c1):
    torch, A, O = env
    rng = np.random.default_rng(0)
    cases = [c1.points, c1.points[:777], rng.integers(-127, 128, (5000, 100)).astype(np.int8),
             rng.standard_normal((3000, 200)).astype(np.float32),
             rng.integers(0, 256, (300, 384)).astype(np.uint8), np.zeros((10, 8), np.uint8)]
    for pts in cases:
        say(f"start vertex {pts.shape} {pts.dtype}")
        assert A.ann_start_vertex(dev(torch, pts)) == O.start_vertex(O.Dataset(pts, 0))


# ------------------------------------------------------------------------------------------
# a5 query search on a graph built by the oracle
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("L", [10, 20, 40, 80, 130, 300])
def test_search_c1_bit_exact(env, c1, c1_oracle, L):
    torch, A, O = env
    ds, g, s = c1_oracle
    gg = A.ann_graph_from_host(g, c1.d, A.U8, A.L2SQ, s)
    pts, qs = dev(torch, c1.points), dev(torch, c1.queries)
    for k in (1, 10, min(L, 70)):
        say(f"search C1 L={L} k={k}")
        ids, dists = A.ann_search(gg, pts, qs, k, L)
        oi, od = O.search_batch(ds, g, s, c1.queries, k, L, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all()
        assert (dists.cpu().numpy() == od).all()


def test_search_tiny_hash_same_result(env, c1, c1_oracle):
    """The visited filter only saves work: a 16-entry table gives the same answers."""
    torch, A, O = env
    ds, g, s = c1_oracle
    pts, qs = dev(torch, c1.points), dev(torch, c1.queries[:200])
    oi, od = O.search_batch(ds, g, s, c1.queries[:200], 10, 40, threads=0)
    # hash_bits is a build option carried by the graph: build two rounds only, then swap rows in
    gg = A.ann_build(pts, c1.R, c1.L, c1.alpha, hash_bits=4, max_rounds=1, start=s)
    g2 = A.ann_graph_from_host(g, c1.d, A.U8, A.L2SQ, s)
    ids, dists = A.ann_search(g2, pts, qs, 10, 40)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    del gg


def test_search_hand_worked_path(env):
    torch, A, O = env
    f = json.load(open(os.path.join(GOLD, "path_search.json")))
    xs = f["xs"]
    n = len(xs)
    pts = np.zeros((n, 4), np.uint8)
    pts[:, 0] = xs
    g = np.full((n, 2), NONE, np.uint32)
    for i in range(n - 1):
        g[i, 0] = i + 1
    q = np.zeros((1, 4), np.uint8)
    q[0, 0] = f["query_x"]
    gg = A.ann_graph_from_host(g, 4, A.U8, A.L2SQ, f["start"])
    ids, dists = A.ann_search(gg, dev(torch, pts), dev(torch, q), f["k"], f["L"])
    assert ids.cpu().numpy()[0].tolist() == f["expect_K"]
    assert dists.cpu().numpy()[0].tolist() == f["expect_K_dists"]


def test_search_unreachable_padding_and_degenerate(env):
    torch, A, O = env
    pts = np.arange(40, dtype=np.uint8).reshape(10, 4)
    g = np.full((10, 3), NONE, np.uint32)
    g[0, 0] = 1
    g[1, :2] = [0, 2]
    gg = A.ann_graph_from_host(g, 4, A.U8, A.L2SQ, 0)
    ids, dists = A.ann_search(gg, dev(torch, pts), dev(torch, pts[5:6]), 5, 8)
    oi, od = O.search_batch(O.Dataset(pts, 0), g, 0, pts[5:6], 5, 8)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    assert oi[0, 3] == NONE and od[0, 3] == np.iinfo(np.int32).max
    # no queries: nothing to do
    A.ann_search(gg, dev(torch, pts), dev(torch, pts[:0]), 1, 1)
    with pytest.raises(A.AnnError):
        A.ann_search(gg, dev(torch, pts), dev(torch, pts[:1]), 9, 8)  # k > L
    with pytest.raises(A.AnnError):
        A.ann_search(gg, dev(torch, pts), dev(torch, pts[:1]), 1, 3000)  # beams end at 2,048


# ------------------------------------------------------------------------------------------
# a3 grouping of reverse edges
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("count,bits", [(0, 5), (1, 5), (63, 3), (64, 7), (1000, 10), (70001, 17), (1 << 20, 20),
                                        (3_000_000, 27)])
def test_sort_edges(env, count, bits):
    torch, A, O = env
    say(f"sort {count} keys on {bits} bits")
    rng = np.random.default_rng(count + bits)
    dst = rng.integers(0, (1 << bits) - 1, count, dtype=np.uint64)
    dst[rng.random(count) < 0.1] = 0xFFFFFFFF  # unused slots
    src = rng.integers(0, 1 << 31, count, dtype=np.uint64)
    keys = (dst << np.uint64(32)) | src
    t = dev(torch, keys.view(np.int64))
    A.ann_sort_edges(t, bits)
    got = t.cpu().numpy().view(np.uint64)
    want = keys[np.argsort(dst & np.uint64((1 << bits) - 1), kind="stable")]
    assert (got == want).all()


# ------------------------------------------------------------------------------------------
# a1-a4 one BatchInsert round on an oracle snapshot, then whole builds
# ------------------------------------------------------------------------------------------
def test_single_rounds_on_oracle_snapshots(env, c1):
    torch, A, O = env
    n = 4000
    pts_h = c1.points[:n]
    ds = O.Dataset(pts_h, 0)
    s = O.start_vertex(ds)
    order = O.insertion_order(n, s, 11)
    theta = 80
    bounds = O.schedule(n - 1, theta).astype(int)
    pts = dev(torch, pts_h)
    for r in (1, 2, 5, 9, 20, len(bounds) - 2):
        say(f"round {r + 1} on the oracle's graph after {r} rounds")
        before, _ = O.build(ds, 32, 64, 1.2, theta=theta, start=s, order=order, max_rounds=r, threads=0)
        after, _ = O.build(ds, 32, 64, 1.2, theta=theta, start=s, order=order, max_rounds=r + 1, threads=0)
        gg = A.ann_graph_from_host(before, c1.d, A.U8, A.L2SQ, s)
        A.ann_insert_batch(gg, pts, order[bounds[r]:bounds[r + 1]], 64, 1.2)
        got = gg.neighbors()
        bad = np.nonzero((got != after).any(1))[0]
        assert len(bad) == 0, f"rows differ: {bad[:10]}"


def test_hand_worked_five_point_build(env):
    torch, A, O = env
    f = json.load(open(os.path.join(GOLD, "five_point_build.json")))
    pts = np.zeros((5, 4), np.int8)
    pts[:, 0] = f["xs"]
    g = A.ann_build(dev(torch, pts), f["R"], f["L"], f["alpha"], batch_cap=f["theta"], start=f["start"],
                    order=np.array(f["order"], np.uint32))
    assert [row_list(r) for r in g.neighbors()] == f["expect_graph"]
    g1 = A.ann_build(dev(torch, pts), f["R"], f["L"], f["alpha"], batch_cap=f["theta"], start=f["start"],
                     order=np.array(f["order"], np.uint32), max_rounds=1)
    assert [row_list(r) for r in g1.neighbors()] == f["expect_after_round_1"]


def test_build_c1_bit_exact_and_deterministic(env, c1, c1_oracle):
    torch, A, O = env
    ds, og, s = c1_oracle
    pts = dev(torch, c1.points)
    say("build C1")
    g = A.ann_build(pts, c1.R, c1.L, c1.alpha, seed=c1.seed, collect_stats=True)
    assert g.info().start == s
    got = g.neighbors()
    bad = np.nonzero((got != og).any(1))[0]
    assert len(bad) == 0, f"{len(bad)} rows differ, first {bad[:5]}"
    st = g.stats()
    ost = O.Stats()
    O.build(ds, c1.R, c1.L, c1.alpha, seed=c1.seed, threads=0, stats=ost)
    assert st["searches"] == ost.searches and st["hops"] == ost.hops
    assert st["reprunes"] == ost.reprunes and st["appends"] == ost.appends and st["edges"] == ost.edges
    assert st["evals"] >= ost.evals  # the lossy filter may repeat evaluations, never skip one
    assert st["rounds"] == ost.rounds == 56
    say("build C1 again")
    g2 = A.ann_build(pts, c1.R, c1.L, c1.alpha, seed=c1.seed)
    assert (g2.neighbors() == got).all()
    # queries on the GPU-built graph
    qs = dev(torch, c1.queries)
    gt, _ = O.brute_force(ds, c1.queries, 10)
    for L in c1.search_L:
        ids, dists = A.ann_search(g, pts, qs, 10, L)
        oi, od = O.search_batch(ds, og, s, c1.queries, 10, L, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
        say(f"  L={L} recall@10={recall_at_k(oi, gt):.4f}")


def test_build_does_not_depend_on_scratch_sizes(env, c1):
    """A visited-list slot of 8 entries forces almost every search through the retry path, and a
    16-entry filter causes many repeated evaluations: the graph must not change."""
    torch, A, O = env
    n = 3000
    pts_h = c1.points[:n]
    ds = O.Dataset(pts_h, 0)
    og, s = O.build(ds, 16, 32, 1.2, seed=3, threads=0)
    pts = dev(torch, pts_h)
    # lists that outgrow their 8-entry slot move to spill chunks on the device ...
    g = A.ann_build(pts, 16, 32, 1.2, seed=3, visited_cap=8, spill_cap=10 ** 6, hash_bits=4, collect_stats=True)
    assert (g.neighbors() == og).all()
    assert g.stats()["restarts"] == 0
    # ... and with (almost) no spill space the build notices at the end, starts over and lets the
    # host redo the searches that did not fit
    g = A.ann_build(pts, 16, 32, 1.2, seed=3, visited_cap=8, spill_cap=1, hash_bits=4, collect_stats=True)
    assert (g.neighbors() == og).all()
    st = g.stats()
    assert st["restarts"] == 1 and st["redone"] > 1000
    # the same through the one-batch entry point, which always checks
    s = O.start_vertex(ds)
    order = O.insertion_order(n, s, 3)
    bounds = O.schedule(n - 1, n // 50).astype(int)
    r = len(bounds) - 3
    before, _ = O.build(ds, 16, 32, 1.2, seed=3, max_rounds=r, threads=0)
    after, _ = O.build(ds, 16, 32, 1.2, seed=3, max_rounds=r + 1, threads=0)
    g3 = A.ann_build(pts, 16, 32, 1.2, seed=3, visited_cap=8, spill_cap=1, max_rounds=r)
    assert (g3.neighbors() == before).all()
    A.ann_insert_batch(g3, pts, order[bounds[r]:bounds[r + 1]], 32, 1.2)
    assert (g3.neighbors() == after).all()


def test_build_hub_segments_spill(env):
    """Many identical points: the start vertex receives a whole batch of reverse edges at once,
    which exceeds the in-LDS candidate buffer of the merge kernel and takes the spill path."""
    torch, A, O = env
    rng = np.random.default_rng(2)
    n = 20000
    pts_h = rng.integers(100, 104, (n, 16)).astype(np.uint8)
    ds = O.Dataset(pts_h, 0)
    s = 0
    order = O.insertion_order(n, s, 1)
    # one huge batch after a few tiny ones: theta = n
    og, _ = O.build(ds, 8, 16, 1.2, theta=n, start=s, order=order, threads=0)
    g = A.ann_build(dev(torch, pts_h), 8, 16, 1.2, batch_cap=n, start=s, order=order)
    assert (g.neighbors() == og).all()


@pytest.mark.parametrize("R,L,alpha,n", [(1, 1, 1.2, 300), (5, 7, 1.0, 500), (70, 100, 1.2, 1500), (130, 140, 2.0, 1200)])
def test_build_odd_parameters(env, c1, R, L, alpha, n):
    torch, A, O = env
    say(f"build R={R} L={L} alpha={alpha} n={n}")
    pts_h = c1.points[:n]
    ds = O.Dataset(pts_h, 0)
    og, s = O.build(ds, R, L, alpha, seed=9, threads=0)
    g = A.ann_build(dev(torch, pts_h), R, L, alpha, seed=9)
    assert g.info().start == s
    assert (g.neighbors() == og).all()


def test_build_tiny_inputs(env):
    torch, A, O = env
    for n in (1, 2, 3, 5):
        pts_h = (np.arange(n * 8, dtype=np.uint8).reshape(n, 8) * 7) % 251
        ds = O.Dataset(pts_h.astype(np.uint8), 0)
        og, s = O.build(ds, 4, 4, 1.2, seed=1)
        g = A.ann_build(dev(torch, pts_h.astype(np.uint8)), 4, 4, 1.2, seed=1)
        assert g.info().start == s and (g.neighbors() == og).all()


def test_bad_arguments(env, c1):
    torch, A, O = env
    pts = dev(torch, c1.points[:100])
    for kw in (dict(R=0, L=8, alpha=1.2), dict(R=8, L=0, alpha=1.2), dict(R=8, L=8, alpha=0.0),
               dict(R=8, L=8, alpha=float("nan")), dict(R=8, L=600, alpha=1.2), dict(R=600, L=8, alpha=1.2)):
        with pytest.raises(A.AnnError):
            A.ann_build(pts, **kw)
    with pytest.raises(A.AnnError):
        A.ann_build(dev(torch, np.tile(c1.points[:100], (1, 5))[:, :520]), 8, 8, 1.2)  # 520-byte rows
    with pytest.raises(A.AnnError):
        A.ann_build(dev(torch, np.ones((100, 6), np.float32)), 8, 8, 1.2)  # f32 rows need d % 4 == 0
    with pytest.raises(A.AnnError):
        A.ann_build(pts, 8, 8, 1.2, metric=A.MIPS)  # inner product on u8
    with pytest.raises(A.AnnError):
        A.ann_build(pts, 8, 8, 1.2, start=100)
    with pytest.raises(A.AnnError):
        A.ann_build(pts, 8, 8, 1.2, start=0, order=np.zeros(99, np.uint32))
    with pytest.raises(A.AnnError):
        A.ann_graph_from_host(np.full((4, 2), 9, np.uint32), 8, A.U8, A.L2SQ, 0)


# ------------------------------------------------------------------------------------------
# other dtypes / metrics
# ------------------------------------------------------------------------------------------
def test_int8_d100_bit_exact(env):
    torch, A, O = env
    w = W.c3(n=6000, nq=300)
    ds = O.Dataset(w.points, 0)
    say("build i8 d=100")
    og, s = O.build(ds, 24, 48, 1.2, seed=2, threads=0)
    pts = dev(torch, w.points)
    g = A.ann_build(pts, 24, 48, 1.2, seed=2)
    assert g.info().start == s
    assert (g.neighbors() == og).all()
    for L in (10, 50, 100):
        ids, dists = A.ann_search(g, pts, dev(torch, w.queries), 10, L)
        oi, od = O.search_batch(ds, og, s, w.queries, 10, L, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()


@pytest.mark.parametrize("d", [1, 4, 6, 20, 30, 36, 64, 100, 256, 300, 512])
def test_u8_other_dimensions(env, d):
    """Rows of any byte length: those that are not a multiple of 16 bytes go through the padded
    copy, queries included."""
    torch, A, O = env
    rng = np.random.default_rng(d)
    n = 1500
    cen = rng.uniform(40, 200, (8, d))
    pts_h = np.clip(np.rint(cen[rng.integers(0, 8, n)] + 15 * rng.standard_normal((n, d))), 0, 255).astype(np.uint8)
    qs_h = np.clip(np.rint(cen[rng.integers(0, 8, 200)] + 15 * rng.standard_normal((200, d))), 0, 255).astype(np.uint8)
    ds = O.Dataset(pts_h, 0)
    og, s = O.build(ds, 12, 24, 1.2, seed=4, threads=0)
    pts = dev(torch, pts_h)
    g = A.ann_build(pts, 12, 24, 1.2, seed=4)
    assert g.info().start == s and (g.neighbors() == og).all()
    for nq in (200, 37):  # the second call reuses the query buffer of the first
        ids, dists = A.ann_search(g, pts, dev(torch, qs_h[:nq]), 5, 30)
        oi, od = O.search_batch(ds, og, s, qs_h[:nq], 5, 30, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # one more batch into a graph given from the host: the padded copy is made on first use
    gg = A.ann_graph_from_host(og, d, A.U8, A.L2SQ, s)
    ids, _ = A.ann_search(gg, pts, dev(torch, qs_h), 5, 30)
    assert (ids.cpu().numpy().view(np.uint32) == O.search_batch(ds, og, s, qs_h, 5, 30, threads=0)[0]).all()


def _float_distance_check(A, O, torch, w, metric, g_rows, s, L):
    """Per-distance tolerance on the GPU's answers: recompute each returned pair in fp64."""
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    gg = A.ann_graph_from_host(g_rows, w.d, A.F32, metric, s)
    ids, dists = A.ann_search(gg, pts, qs, 10, L)
    ids = ids.cpu().numpy().view(np.uint32)
    dists = dists.cpu().numpy()
    assert (ids != NONE).all()
    P = w.points[ids].astype(np.float64)              # nq x k x d
    Q = w.queries.astype(np.float64)[:, None, :]
    if metric == A.L2SQ:
        ref = ((P - Q) ** 2).sum(-1)
        scale = np.abs(ref)
    else:
        ref = -(P * Q).sum(-1)
        scale = np.abs(P * Q).sum(-1)
    err = np.abs(dists.astype(np.float64) - ref)
    assert (err <= 1e-5 * scale + 1e-30).all(), f"max rel err {np.max(err / (scale + 1e-30))}"
    big = np.abs(ref) >= 0.05
    if big.any():
        assert (err[big] <= 1e-5 * np.abs(ref[big])).all()
    assert (np.diff(dists, axis=1) >= 0).all()
    return ids, dists


@pytest.mark.parametrize("metric,alpha", [(0, 1.2), (1, 1.0)])
def test_f32_distances_and_recall(env, metric, alpha):
    torch, A, O = env
    w = W.c4(n=8000, nq=400)
    ds = O.Dataset(w.points, metric)
    say(f"f32 metric={metric}: oracle build")
    og, s = O.build(ds, 32, 64, alpha, seed=1, threads=0)
    gt, _ = O.brute_force(ds, w.queries, 10)
    # same graph on both sides: answers agree up to near-ties in fp32
    ids, dists = _float_distance_check(A, O, torch, w, metric, og, s, 64)
    oi, od = O.search_batch(ds, og, s, w.queries, 10, 64, threads=0)
    assert abs(recall_at_k(ids, gt) - recall_at_k(oi, gt)) <= 0.002
    assert (ids == oi).mean() > 0.99
    # GPU-built graph: recall within 0.002 of the oracle-built graph at equal L
    say("  GPU build")
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    g = A.ann_build(pts, 32, 64, alpha, seed=1, metric=metric)
    assert g.info().start == s
    rows = g.neighbors()
    deg = (rows != NONE).sum(1)
    assert deg.max() <= 32 and deg[np.arange(len(deg)) != s].min() >= 1
    same_rows = (rows == og).all(1).mean()
    say(f"  rows identical to the oracle's: {same_rows:.5f}")
    assert same_rows >= 0.99  # near-ties in fp32 may flip a few (measured: all identical)
    for L in (20, 64):
        gi, _ = A.ann_search(g, pts, qs, 10, L)
        oi, _ = O.search_batch(ds, og, s, w.queries, 10, L, threads=0)
        r_g = recall_at_k(gi.cpu().numpy().view(np.uint32), gt)
        r_o = recall_at_k(oi, gt)
        say(f"  L={L} recall gpu={r_g:.4f} oracle={r_o:.4f}")
        assert abs(r_g - r_o) <= 0.002
    g2 = A.ann_build(pts, 32, 64, alpha, seed=1, metric=metric)
    assert (g2.neighbors() == rows).all()


# ------------------------------------------------------------------------------------------
# full size (the benchmark's workload and launch configuration), on samples the oracle can do
# ------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def c2_full(env):
    torch, A, O = env
    w = W.c2()
    pts = dev(torch, w.points)
    g = A.ann_build(pts, w.R, w.L, w.alpha, seed=w.seed, collect_stats=True)
    g.build_stats = g.stats()  # before any query adds to the counters
    return w, pts, g


def test_c2_full_size_build_sampled_against_oracle(env, c2_full):
    """The graph before the last batch comes from a GPU build stopped one batch early; the oracle
    and the GPU both insert the same 3,000 points of the last batch into it: identical rows."""
    torch, A, O = env
    w, pts, g = c2_full
    rounds = int(g.info().rounds)
    snap = A.ann_build(pts, w.R, w.L, w.alpha, seed=w.seed, max_rounds=rounds - 1)
    rows = snap.neighbors()
    s = int(snap.info().start)
    ds = O.Dataset(w.points, 0)
    assert s == O.start_vertex(ds)
    order = O.insertion_order(w.n, s, w.seed)
    bounds = O.schedule(w.n - 1, w.theta).astype(np.int64)
    assert len(bounds) - 1 == rounds
    batch = order[bounds[rounds - 1]:bounds[rounds]][:3000]
    say(f"oracle inserts {len(batch)} points into the {int(bounds[rounds - 1]) + 1}-point graph")
    og = rows.copy()
    O.batch_insert(ds, og, s, batch, w.L, w.alpha, threads=0)
    A.ann_insert_batch(snap, pts, batch, w.L, w.alpha)
    gg = snap.neighbors()
    changed = np.nonzero((og != rows).any(1))[0]
    assert len(changed) > len(batch)  # the batch's own rows and the rows that took reverse edges
    bad = np.nonzero((gg != og).any(1))[0]
    assert len(bad) == 0, f"rows differ: {bad[:10]}"


def test_c2_full_size_queries_against_oracle(env, c2_full):
    torch, A, O = env
    w, pts, g = c2_full
    rows = g.neighbors()
    s = int(g.info().start)
    ds = O.Dataset(w.points, 0)
    qs_h = w.queries[:300]
    qs = dev(torch, qs_h)
    for L in (10, 50, 200):
        say(f"300 queries on the full graph, L={L}")
        ids, dists = A.ann_search(g, pts, qs, 10, L)
        oi, od = O.search_batch(ds, rows, s, qs_h, 10, L, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all()
        assert (dists.cpu().numpy().view(np.int32) == od.view(np.int32)).all()


def test_c2_full_size_invariants(env, c2_full):
    """Properties that hold at any size: degree bounds, rows are compact lists of valid ids without
    self loops or repeats, the counters add up, and a second build gives the same bytes."""
    torch, A, O = env
    w, pts, g = c2_full
    rows = g.neighbors()
    n = w.n
    valid = rows != NONE
    deg = valid.sum(1)
    assert deg.max() <= w.R and deg.min() >= 1
    # valid ids come first in every row
    assert (valid[:, :-1] >= valid[:, 1:]).all()
    assert rows[valid].max() < n
    assert not (rows == np.arange(n, dtype=np.uint32)[:, None]).any()
    srt = np.sort(rows, axis=1)
    assert not ((srt[:, 1:] == srt[:, :-1]) & (srt[:, 1:] != NONE)).any()
    st = g.build_stats
    assert st["searches"] == n - 1 and st["prunes"] == n - 1 and st["restarts"] == 0
    g2 = A.ann_build(pts, w.R, w.L, w.alpha, seed=w.seed)
    assert (g2.neighbors() == rows).all()


def test_c2_full_size_every_filter_layout_gives_the_same_graph(env, c2_full):
    """The visited filter only saves work.  At a million points the default table holds 16-bit
    tags; 8 buckets force 21-bit tags (20 id bits - 3) and 4 buckets with ids handed in as a
    larger graph would; a tiny table also makes nearly every candidate come back, which exercises
    the duplicate handling.  Checked on a partial build to keep it short."""
    torch, A, O = env
    w, pts, g = c2_full
    ref = A.ann_build(pts, w.R, w.L, w.alpha, seed=w.seed, max_rounds=22).neighbors()
    for hb in (5, 7, 12):
        say(f"partial build with hash_bits={hb}")
        got = A.ann_build(pts, w.R, w.L, w.alpha, seed=w.seed, max_rounds=22, hash_bits=hb).neighbors()
        assert (got == ref).all()
    qs = dev(torch, w.queries[:500])
    ids0, d0 = A.ann_search(g, pts, qs, 10, 40)
    g5 = A.ann_build(pts, w.R, w.L, w.alpha, seed=w.seed, hash_bits=5)
    assert (g5.neighbors() == g.neighbors()).all()
    ids1, d1 = A.ann_search(g5, pts, qs, 10, 40)
    assert (ids0 == ids1).all() and (d0 == d1).all()


# ------------------------------------------------------------------------------------------
# the (1 + eps) rule of the search (Sec. 4.5)
# ------------------------------------------------------------------------------------------
def test_search_eps_hand_worked_path(env):
    torch, A, O = env
    f = json.load(open(os.path.join(GOLD, "eps_path.json")))
    for dtype, code in ((np.uint8, A.U8), (np.float32, A.F32)):
        xs = f["xs"]
        n = len(xs)
        pts = np.zeros((n, 4), dtype)
        pts[:, 0] = xs
        g = np.full((n, 2), NONE, np.uint32)
        for i in range(n):
            nb = [j for j in (i - 1, i + 1) if 0 <= j < n]
            g[i, :len(nb)] = nb
        q = np.zeros((1, 4), dtype)
        q[0, 0] = f["query_x"]
        gg = A.ann_graph_from_host(g, 4, code, A.L2SQ, f["start"])
        ds = O.Dataset(pts, 0)
        for c in f["cases"]:
            ids, dists = A.ann_search(gg, dev(torch, pts), dev(torch, q), c["k"], f["L"], eps=c["eps"])
            assert ids.cpu().numpy().view(np.uint32)[0].tolist() == c["expect_K"], (dtype, c)
            oi, od = O.search_batch(ds, g, f["start"], q, c["k"], f["L"], eps=c["eps"])
            assert (dists.cpu().numpy() == od).all()


@pytest.mark.parametrize("eps", [0.0, 0.02, 0.1, 0.25, 3.0])
def test_search_eps_c1_bit_exact(env, c1, c1_oracle, eps):
    torch, A, O = env
    ds, g, s = c1_oracle
    gg = A.ann_graph_from_host(g, c1.d, A.U8, A.L2SQ, s)
    pts, qs = dev(torch, c1.points), dev(torch, c1.queries)
    for L, k in ((10, 10), (40, 10), (130, 10), (64, 1), (300, 70)):
        say(f"search C1 eps={eps} L={L} k={k}")
        ids, dists = A.ann_search_eps(gg, pts, qs, k, L, eps)
        oi, od = O.search_batch(ds, g, s, c1.queries, k, L, threads=0, eps=eps)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all()
        assert (dists.cpu().numpy() == od).all()
    # a negative eps is plain ann_search
    a0 = A.ann_search(gg, pts, qs, 10, 40)
    a1 = A.ann_search_eps(gg, pts, qs, 10, 40, -1.0)
    assert (a0[0] == a1[0]).all() and (a0[1] == a1[1]).all()
    with pytest.raises(A.AnnError):
        A.ann_search_eps(gg, pts, qs, 10, 40, float("nan"))
    with pytest.raises(A.AnnError):
        A.ann_search_eps(gg, pts, qs, 10, 40, 1e9)


def test_search_eps_c2_full_size(env, c2_full):
    """Full size: 300 queries against the oracle, and the rule really saves hops."""
    torch, A, O = env
    w, pts, g = c2_full
    rows = g.neighbors()
    s = int(g.info().start)
    ds = O.Dataset(w.points, 0)
    qs_h = w.queries[:300]
    qs = dev(torch, qs_h)
    for L, eps in ((30, 0.05), (100, 0.1), (200, 0.25)):
        ids, dists = A.ann_search_eps(g, pts, qs, 10, L, eps)
        so, sp = O.Stats(), O.Stats()
        oi, od = O.search_batch(ds, rows, s, qs_h, 10, L, threads=0, eps=eps, stats=sp)
        O.search_batch(ds, rows, s, qs_h, 10, L, threads=0, stats=so)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all()
        assert (dists.cpu().numpy().view(np.int32) == od.view(np.int32)).all()
        assert sp.hops < so.hops


# ------------------------------------------------------------------------------------------
# streaming insertion of new points (ann_insert_points): BatchInsert of Alg. 3 after the build
# ------------------------------------------------------------------------------------------
def test_insert_points_c1_bit_exact(env, c1):
    """Build over the first 6,000 points, stream the rest in with two calls: rows, start vertex
    and query answers identical to the oracle's at every stage; the capacity of the row array
    (grown on demand, or reserved in advance) does not show."""
    torch, A, O = env
    cuts = (6000, 8500, c1.n)
    pts = dev(torch, c1.points)
    og, s = O.build(O.Dataset(c1.points[:cuts[0]], 0), c1.R, c1.L, c1.alpha, seed=c1.seed, threads=0)
    g = A.ann_build(pts[:cuts[0]], c1.R, c1.L, c1.alpha, seed=c1.seed)
    g2 = A.ann_build(pts[:cuts[0]], c1.R, c1.L, c1.alpha, seed=c1.seed)
    A.ann_graph_reserve(g2, c1.n)
    assert g.info().start == s and (g.neighbors() == og).all() and (g2.neighbors() == og).all()
    for seed, n_tot in ((3, cuts[1]), (4, cuts[2])):
        say(f"insert points up to {n_tot}")
        ds = O.Dataset(c1.points[:n_tot], 0)
        og = O.insert_points(ds, og, s, c1.L, c1.alpha, seed=seed, threads=0)
        for gg in (g, g2):
            A.ann_insert_points(gg, pts[:n_tot], c1.L, c1.alpha, seed=seed)
            assert gg.info().n == n_tot and gg.info().start == s
            rows = gg.neighbors()
            assert rows.shape == og.shape
            bad = np.nonzero((rows != og).any(1))[0]
            assert len(bad) == 0, f"rows differ: {bad[:10]}"
        ids, dists = A.ann_search(g, pts[:n_tot], dev(torch, c1.queries), 10, 40)
        oi, od = O.search_batch(ds, og, s, c1.queries, 10, 40, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # nothing to add: nothing happens
    A.ann_insert_points(g, pts, c1.L, c1.alpha, seed=9)
    assert (g.neighbors() == og).all()


def test_insert_points_continues_a_build(env, c1):
    """A build cut at a batch boundary and continued by ann_insert_points is the one-shot build
    (same start vertex, theta and order), also when the remainder arrives in two calls that
    each end on a boundary."""
    torch, A, O = env
    n, theta = 5000, 300
    pts = dev(torch, c1.points[:n])
    order = np.arange(1, n, dtype=np.uint32)
    whole = A.ann_build(pts, 16, 32, 1.2, batch_cap=theta, start=0, order=order).neighbors()
    b = O.schedule(n - 1, theta).astype(np.int64)
    r1, r2 = 9, 14
    n1, n2 = int(b[r1]) + 1, int(b[r2]) + 1
    g = A.ann_build(pts[:n1], 16, 32, 1.2, batch_cap=theta, start=0, order=order[:n1 - 1])
    A.ann_insert_points(g, pts[:n2], 32, 1.2, batch_cap=theta, order=order[n1 - 1:n2 - 1])
    A.ann_insert_points(g, pts, 32, 1.2, batch_cap=theta, order=order[n2 - 1:])
    assert (g.neighbors() == whole).all()
    # max_rounds stops early: the rows of the points not yet reached stay empty
    g = A.ann_build(pts[:n1], 16, 32, 1.2, batch_cap=theta, start=0, order=order[:n1 - 1])
    A.ann_insert_points(g, pts, 32, 1.2, batch_cap=theta, order=order[n1 - 1:], max_rounds=2)
    rows = g.neighbors()
    assert (rows[int(b[r1 + 2]) + 1:] == NONE).all() and (rows[n1:int(b[r1 + 2]) + 1, 0] != NONE).all()


def test_insert_points_padded_rows_and_moved_arrays(env):
    """100-byte int8 rows (the kernels read a padded copy that has to follow the graph): the new
    points arrive in the array the graph was built over (the copy is made anew when it has to
    grow, extended when there is room) and then in a fresh copy of the points."""
    torch, A, O = env
    w = W.c3(n=6000, nq=200)
    og, s = O.build(O.Dataset(w.points[:3000], 0), 24, 48, 1.2, seed=2, threads=0)
    pts = dev(torch, w.points)
    g = A.ann_build(pts[:3000], 24, 48, 1.2, seed=2)
    assert (g.neighbors() == og).all()
    A.ann_graph_reserve(g, 6000)
    for seed, n_tot in ((5, 4000), (6, 5000)):
        og = O.insert_points(O.Dataset(w.points[:n_tot], 0), og, s, 48, 1.2, seed=seed, threads=0)
        A.ann_insert_points(g, pts[:n_tot], 48, 1.2, seed=seed)
        assert (g.neighbors() == og).all()
    moved = dev(torch, w.points.copy())
    assert moved.data_ptr() != pts.data_ptr()
    ds = O.Dataset(w.points, 0)
    og = O.insert_points(ds, og, s, 48, 1.2, seed=7, theta=100, threads=0)
    A.ann_insert_points(g, moved, 48, 1.2, seed=7, batch_cap=100)
    assert (g.neighbors() == og).all()
    ids, dists = A.ann_search(g, moved, dev(torch, w.queries), 10, 50)
    oi, od = O.search_batch(ds, og, s, w.queries, 10, 50, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()


def test_insert_points_f32(env):
    torch, A, O = env
    w = W.c4(n=8000, nq=400)
    n0 = 5000
    ds = O.Dataset(w.points, 1)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    g = A.ann_build(pts[:n0], 32, 64, 1.0, seed=1, metric=A.MIPS)
    s = int(g.info().start)
    head = g.neighbors()
    # the oracle continues from the GPU's graph, so that only this call's arithmetic differs
    og = O.insert_points(ds, head, s, 64, 1.0, seed=7, threads=0)
    A.ann_insert_points(g, pts, 64, 1.0, seed=7)
    rows = g.neighbors()
    deg = (rows != NONE).sum(1)
    assert deg.max() <= 32 and deg[np.arange(len(deg)) != s].min() >= 1
    same_rows = (rows == og).all(1).mean()
    say(f"  rows identical to the oracle's: {same_rows:.5f}")
    assert same_rows >= 0.99  # near-ties in fp32 may flip a few rows
    gt, _ = O.brute_force(ds, w.queries, 10)
    gi, _ = A.ann_search(g, pts, qs, 10, 64)
    oi, _ = O.search_batch(ds, og, s, w.queries, 10, 64, threads=0)
    r_g, r_o = recall_at_k(gi.cpu().numpy().view(np.uint32), gt), recall_at_k(oi, gt)
    say(f"  recall after streaming insertion: gpu={r_g:.4f} oracle={r_o:.4f}")
    assert abs(r_g - r_o) <= 0.002


def test_insert_points_bad_arguments(env, c1):
    torch, A, O = env
    pts = dev(torch, c1.points[:3000])
    g = A.ann_build(pts[:2000], 8, 16, 1.2)
    rows = g.neighbors()
    with pytest.raises(A.AnnError):
        A.ann_insert_points(g, pts[:1500], 16, 1.2)                      # fewer points than the graph holds
    with pytest.raises(A.AnnError):
        A.ann_insert_points(g, pts, 0, 1.2)                              # L
    with pytest.raises(A.AnnError):
        A.ann_insert_points(g, pts, 16, -1.0)                            # alpha
    bad = np.arange(2000, 3000, dtype=np.uint32)
    bad[5] = 1999                                                        # an id the graph already holds
    with pytest.raises(A.AnnError):
        A.ann_insert_points(g, pts, 16, 1.2, order=bad)
    bad[5] = 2006                                                        # a new id twice
    with pytest.raises(A.AnnError):
        A.ann_insert_points(g, pts, 16, 1.2, order=bad)
    assert g.info().n == 2000 and (g.neighbors() == rows).all()          # refused calls change nothing


def test_insert_points_c2_full_size(env):
    """At the benchmark's size and launch configuration: a graph over 995,000 points takes the
    last 5,000 (one batch, theta = 20,000); the oracle does the same on a copy of that graph."""
    torch, A, O = env
    w = W.c2()
    n0 = w.n - 5000
    pts = dev(torch, w.points)
    g = A.ann_build(pts[:n0], w.R, w.L, w.alpha, seed=w.seed)
    s = int(g.info().start)
    head = g.neighbors()
    ds = O.Dataset(w.points, 0)
    say("oracle streams 5,000 points into the 995,000-point graph")
    st = O.Stats()
    og = O.insert_points(ds, head, s, w.L, w.alpha, seed=11, threads=0, stats=st)
    assert st.rounds == 1
    A.ann_insert_points(g, pts, w.L, w.alpha, seed=11)
    rows = g.neighbors()
    assert ((og[:n0] != head).any(1)).sum() > 5000  # many old rows took reverse edges
    bad = np.nonzero((rows != og).any(1))[0]
    assert len(bad) == 0, f"rows differ: {bad[:10]}"
    ids, dists = A.ann_search(g, pts, dev(torch, w.queries[:300]), 10, 40)
    oi, od = O.search_batch(ds, og, s, w.queries[:300], 10, 40, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()


# ------------------------------------------------------------------------------------------
# layered index (Sec. 4.2, ParlayHNSW)
# ------------------------------------------------------------------------------------------
def _hnsw_layers_global(h, n):
    """The library's layers as n x degree arrays of point ids, the oracle's format."""
    hi = h.info()
    out = []
    for l in range(hi.top + 1):
        ids, rows = h.layer(l)
        full = np.full((n, rows.shape[1]), NONE, np.uint32)
        full[ids] = rows
        out.append((ids, full))
    return out


def _check_hnsw_against(h, oh, n):
    hi = h.info()
    assert hi.top == oh.top and hi.entry == oh.entry
    assert (h.levels() == oh.level).all()
    for l, (ids, full) in enumerate(_hnsw_layers_global(h, n)):
        assert (ids == np.flatnonzero(oh.level >= l)).all()
        bad = np.nonzero((full != oh.layers[l]).any(1))[0]
        assert len(bad) == 0, f"layer {l}: rows differ: {bad[:10]}"


@pytest.mark.parametrize("m,efc,alpha", [(16, 64, 1.0), (4, 20, 1.2), (32, 128, 0.82)])
def test_hnsw_c1_bit_exact(env, c1, m, efc, alpha):
    torch, A, O = env
    ds = O.Dataset(c1.points, 0)
    say(f"layered index m={m} efc={efc} alpha={alpha}: oracle build")
    oh = O.hnsw_build(ds, m, efc, alpha, seed=5, threads=0)
    pts, qs = dev(torch, c1.points), dev(torch, c1.queries)
    h = A.ann_hnsw_build(pts, m, efc, alpha, seed=5)
    assert oh.top >= 2
    _check_hnsw_against(h, oh, c1.n)
    for L, k, eps in ((10, 10, -1.0), (40, 10, -1.0), (1, 1, -1.0), (130, 20, -1.0), (40, 10, 0.1), (40, 10, 0.0)):
        ids, dists = A.ann_hnsw_search(h, pts, qs, k, L, eps=eps)
        oi, od, _ = O.hnsw_search_batch(ds, oh, c1.queries, k, L, eps=eps, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # deterministic
    h2 = A.ann_hnsw_build(pts, m, efc, alpha, seed=5)
    for (_, a), (_, b) in zip(_hnsw_layers_global(h, c1.n), _hnsw_layers_global(h2, c1.n)):
        assert (a == b).all()


def test_hnsw_one_layer_is_the_flat_graph(env, c1):
    torch, A, O = env
    n, m = 4000, 12
    pts = dev(torch, c1.points[:n])
    h = A.ann_hnsw_build(pts, m, 48, 1.2, seed=3, level=np.zeros(n, np.uint32))
    g = A.ann_build(pts, 2 * m, 48, 1.2, seed=3, start=0)
    assert h.info().top == 0 and h.info().entry == 0
    assert (h.layer(0)[1] == g.neighbors()).all()
    qs = dev(torch, c1.queries)
    a, b = A.ann_hnsw_search(h, pts, qs, 10, 30), A.ann_search(g, pts, qs, 10, 30)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


def test_hnsw_given_levels_order_and_partial_builds(env, c1):
    """Levels and order given by the caller (a tall, thin hierarchy), stopped after a few batches:
    identical to the oracle's at every stop."""
    torch, A, O = env
    n, m = 3000, 6
    rng = np.random.default_rng(1)
    level = rng.geometric(0.5, n).astype(np.uint32) - 1
    level[level > 9] = 9
    entry = int(np.flatnonzero(level == level.max())[0])
    order = rng.permutation(np.delete(np.arange(n, dtype=np.uint32), entry))
    ds = O.Dataset(c1.points[:n], 0)
    pts = dev(torch, c1.points[:n])
    for rounds in (1, 4, 12, 0):
        oh = O.hnsw_build(ds, m, 30, 1.1, theta=100, level=level, order=order, max_rounds=rounds, threads=0)
        h = A.ann_hnsw_build(pts, m, 30, 1.1, batch_cap=100, level=level, order=order, max_rounds=rounds)
        _check_hnsw_against(h, oh, n)


def test_hnsw_padded_int8_and_f32(env):
    torch, A, O = env
    w = W.c3(n=6000, nq=300)
    ds = O.Dataset(w.points, 0)
    oh = O.hnsw_build(ds, 12, 48, 1.0, seed=2, threads=0)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    h = A.ann_hnsw_build(pts, 12, 48, 1.0, seed=2)
    _check_hnsw_against(h, oh, w.n)
    ids, dists = A.ann_hnsw_search(h, pts, qs, 10, 50)
    oi, od, _ = O.hnsw_search_batch(ds, oh, w.queries, 10, 50, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()

    w = W.c4(n=8000, nq=400)
    ds = O.Dataset(w.points, 1)
    oh = O.hnsw_build(ds, 16, 64, 1.0, seed=1, threads=0)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    h = A.ann_hnsw_build(pts, 16, 64, 1.0, seed=1, metric=A.MIPS)
    assert h.info().top == oh.top and h.info().entry == oh.entry
    same = [(full == oh.layers[l]).all(1).mean() for l, (_, full) in enumerate(_hnsw_layers_global(h, w.n))]
    say(f"  rows identical to the oracle's, per layer: {same}")
    assert min(same) >= 0.99  # near-ties in fp32 may flip a few rows
    gt, _ = O.brute_force(ds, w.queries, 10)
    gi, _ = A.ann_hnsw_search(h, pts, qs, 10, 64)
    oi, _, _ = O.hnsw_search_batch(ds, oh, w.queries, 10, 64, threads=0)
    r_g, r_o = recall_at_k(gi.cpu().numpy().view(np.uint32), gt), recall_at_k(oi, gt)
    say(f"  recall gpu={r_g:.4f} oracle={r_o:.4f}")
    assert abs(r_g - r_o) <= 0.002


def test_hnsw_bad_arguments(env, c1):
    torch, A, O = env
    pts = dev(torch, c1.points[:500])
    for kw in (dict(m=1, efc=8, alpha=1.0), dict(m=300, efc=8, alpha=1.0), dict(m=8, efc=0, alpha=1.0),
               dict(m=8, efc=8, alpha=0.0)):
        with pytest.raises(A.AnnError):
            A.ann_hnsw_build(pts, **kw)
    with pytest.raises(A.AnnError):
        A.ann_hnsw_build(pts, 8, 16, 1.0, level=np.full(500, 64, np.uint32))
    with pytest.raises(A.AnnError):
        A.ann_hnsw_build(pts, 8, 16, 1.0, order=np.zeros(499, np.uint32))
    h = A.ann_hnsw_build(pts, 8, 16, 1.0)
    qs = dev(torch, c1.queries[:10])
    with pytest.raises(A.AnnError):
        A.ann_hnsw_search(h, pts, qs, 10, 5)
    with pytest.raises(A.AnnError):
        h.layer(h.info().top + 1)
    # a single point, and two
    for n in (1, 2):
        h = A.ann_hnsw_build(pts[:n], 4, 8, 1.0)
        ids, _ = A.ann_hnsw_search(h, pts[:n], qs, 1, 4)
        assert (ids.cpu().numpy() < n).all()


def test_hnsw_c2_full_size_last_batch_against_oracle(env):
    """The benchmark's size and launch configuration (m = 32, efc = 128, alpha = 0.82, the
    appendix's setting for the 128-d uint8 set): the index before the last batch comes from a GPU
    build stopped one batch early; the oracle inserts that batch into a copy of it, the GPU
    finishes its own build; every layer identical, and so are query answers."""
    torch, A, O = env
    w = W.c2()
    pts, qs = dev(torch, w.points), dev(torch, w.queries[:300])
    m, efc, alpha = 32, 128, 0.82
    full = A.ann_hnsw_build(pts, m, efc, alpha, seed=w.seed)
    rounds = int(full.info().rounds)
    part = A.ann_hnsw_build(pts, m, efc, alpha, seed=w.seed, max_rounds=rounds - 1)
    hi = part.info()
    level = part.levels()
    oh = O.Hnsw(m, level, [f for _, f in _hnsw_layers_global(part, w.n)], hi.entry)
    order = O.insertion_order(w.n, hi.entry, w.seed)
    bounds = O.schedule(w.n - 1, w.theta).astype(np.int64)
    assert len(bounds) - 1 == rounds
    batch = order[bounds[rounds - 1]:]
    ds = O.Dataset(w.points, 0)
    say(f"oracle inserts the last batch ({len(batch)} points) into the {hi.top + 1}-layer index")
    O.hnsw_insert_batch(ds, oh, batch, efc, alpha, threads=0)
    _check_hnsw_against(full, oh, w.n)
    ids, dists = A.ann_hnsw_search(full, pts, qs, 10, 40)
    oi, od, _ = O.hnsw_search_batch(ds, oh, w.queries[:300], 10, 40, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()


def test_hnsw_search_worked_by_hand(env):
    torch, A, O = env
    g = json.load(open(os.path.join(GOLD, "hnsw_descent.json")))
    xs, m = g["xs"], g["m"]
    n = len(xs)
    layers = []
    for l in range(len(g["layers"])):
        rows = np.full((n, 2 * m if l == 0 else m), NONE, np.uint32)
        for v, nb in g["layers"][str(l)].items():
            rows[int(v), :len(nb)] = nb
        layers.append(rows)
    for dtype, d in ((np.uint8, 16), (np.uint8, 4), (np.float32, 4)):
        pts = np.zeros((n, d), dtype)
        pts[:, 0] = xs
        h = A.ann_hnsw_from_host(dev(torch, pts), m, g["level"], g["entry"], layers)
        for c in g["cases"]:
            q = np.zeros((1, d), dtype)
            q[0, 0] = c["query_x"]
            ids, dists = A.ann_hnsw_search(h, dev(torch, pts), dev(torch, q), g["k"], g["L"])
            assert ids.cpu().numpy()[0].tolist() == c["expect_ids"]
            assert dists.cpu().numpy()[0].tolist() == c["expect_dists"]
        # the layers come back as they went in
        for l, rows in enumerate(layers):
            ids_l, rows_l = h.layer(l)
            assert (ids_l == np.flatnonzero(np.array(g["level"]) >= l)).all() and (rows_l == rows[ids_l]).all()


def test_hnsw_from_host_round_trip(env, c1):
    """An index built by the oracle, handed to the library: same answers as the oracle's search,
    for every beam width (the walk down runs in a kernel of its own, with no visited set)."""
    torch, A, O = env
    n = 6000
    ds = O.Dataset(c1.points[:n], 0)
    oh = O.hnsw_build(ds, 5, 24, 1.2, seed=8, threads=0)
    assert oh.top >= 3
    pts, qs = dev(torch, c1.points[:n]), dev(torch, c1.queries)
    h = A.ann_hnsw_from_host(pts, 5, oh.level, oh.entry, oh.layers)
    _check_hnsw_against(h, oh, n)
    for L, k in ((1, 1), (8, 5), (50, 10)):
        ids, dists = A.ann_hnsw_search(h, pts, qs, k, L)
        oi, od, _ = O.hnsw_search_batch(ds, oh, c1.queries, k, L, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    bad = [a.copy() for a in oh.layers]
    bad[1][np.flatnonzero(oh.level >= 1)[0], 0] = int(np.flatnonzero(oh.level == 0)[0])  # not on layer 1
    with pytest.raises(A.AnnError):
        A.ann_hnsw_from_host(pts, 5, oh.level, oh.entry, bad)
    with pytest.raises(A.AnnError):
        A.ann_hnsw_from_host(pts, 5, oh.level, int(np.flatnonzero(oh.level == 0)[0]), oh.layers)


# ------------------------------------------------------------------------------------------
# clustering-based builder (Sec. 3.2 and 4.3, ParlayHCNNG)
# ------------------------------------------------------------------------------------------
def _oracle_tree_pairs(O, ds, Ls, s, l, seed, tree):
    perm, off = O.hcnng_tree(ds, Ls, seed, tree)
    pairs = [O.hcnng_leaf(ds, perm[off[j]:off[j + 1]], s, l) for j in range(len(off) - 1)]
    return perm, off, np.concatenate(pairs) if pairs else np.zeros((0, 2), np.uint32)


@pytest.mark.parametrize("n,Ls,s,l", [(3000, 100, 3, 10), (2000, 37, 2, 4), (1500, 1024, 3, 10), (700, 64, 1, 16),
                                      (900, 2, 3, 10), (1200, 150, 200, 16)])
def test_hcnng_one_tree_bit_exact(env, c1, n, Ls, s, l):
    """Cluster tree, leaves and every leaf's accepted pairs, in acceptance order."""
    torch, A, O = env
    pts_h = c1.points[:n]
    ds = O.Dataset(pts_h, 0)
    pts = dev(torch, pts_h)
    for tree in (0, 3):
        say(f"cluster tree {tree}: n={n} Ls={Ls} s={s} l={l}")
        perm, off, pairs = A.ann_hcnng_tree_edges(pts, Ls, s, l, 5, tree)
        operm, ooff, opairs = _oracle_tree_pairs(O, ds, Ls, s, l, 5, tree)
        assert (off == ooff).all() and (perm == operm).all()
        assert pairs.shape == opairs.shape and (pairs == opairs).all()


def test_hcnng_equal_points_and_tiny_inputs(env):
    torch, A, O = env
    same = np.full((300, 16), 7, np.uint8)
    same[100:] = 9
    perm, off, pairs = A.ann_hcnng_tree_edges(dev(torch, same), 16, 3, 10, 1, 0)
    operm, ooff, opairs = _oracle_tree_pairs(O, O.Dataset(same, 0), 16, 3, 10, 1, 0)
    assert (off == ooff).all() and (perm == operm).all() and (pairs == opairs).all()
    for n in (1, 2, 3):
        pts_h = (np.arange(n * 8, dtype=np.uint8).reshape(n, 8) * 7) % 251
        perm, off, pairs = A.ann_hcnng_tree_edges(dev(torch, pts_h), 2, 3, 10, 1, 0)
        operm, ooff, opairs = _oracle_tree_pairs(O, O.Dataset(pts_h, 0), 2, 3, 10, 1, 0)
        assert (off == ooff).all() and (perm == operm).all() and (pairs == opairs).all()


def test_hcnng_leaf_tiles_allocated_again(env, c1, monkeypatch):
    """The buffer of leaf tiles starts too small (one tile) and is allocated again for the group."""
    torch, A, O = env
    monkeypatch.setenv("ANN_HCNNG_FEW_TILES", "1")
    n, T, Ls, s, l, R = 2000, 5, 90, 3, 10, 24
    pts_h = c1.points[:n]
    og = O.hcnng_build(O.Dataset(pts_h, 0), T, Ls, s, l, R, 1.2, seed=3, threads=0)
    say("clustering-based build with the tile buffer grown on demand")
    g = A.ann_hcnng_build(dev(torch, pts_h), T, Ls, s, l, R, 1.2, seed=3)
    assert (g.neighbors() == og).all()


@pytest.mark.parametrize("signed", [False, True])
def test_hcnng_largest_distances(env, signed):
    """Rows of 128 bytes at the ends of the value range: squared distances up to 128 * 255^2, the
    largest the nearest-neighbour kernel's packed (distance, candidate) keys have to hold."""
    torch, A, O = env
    rng = np.random.default_rng(11)
    n, d = 1400, 128
    lo, hi = (-128, 127) if signed else (0, 255)
    pts_h = rng.integers(lo, hi + 1, (n, d)).astype(np.int8 if signed else np.uint8)
    kind = rng.integers(0, 4, n)
    pts_h[kind == 0] = lo  # many equal rows at either end, and rows that mix the two ends
    pts_h[kind == 1] = hi
    mixed = np.nonzero(kind == 2)[0]
    pts_h[mixed] = np.where(rng.integers(0, 2, (len(mixed), d)) == 1, hi, lo).astype(pts_h.dtype)
    ds = O.Dataset(pts_h, 0)
    say(f"largest distances, signed={signed}")
    perm, off, pairs = A.ann_hcnng_tree_edges(dev(torch, pts_h), 700, 3, 10, 3, 0)
    operm, ooff, opairs = _oracle_tree_pairs(O, ds, 700, 3, 10, 3, 0)
    assert (off == ooff).all() and (perm == operm).all()
    assert pairs.shape == opairs.shape and (pairs == opairs).all()


@pytest.mark.parametrize("n,T,Ls,s,l,R,alpha", [(3000, 6, 120, 3, 10, 20, 1.2), (2500, 12, 60, 3, 10, 8, 1.0),
                                                (2000, 3, 500, 5, 16, 64, 1.2), (1500, 40, 30, 3, 5, 32, 1.2)])
def test_hcnng_build_bit_exact(env, c1, n, T, Ls, s, l, R, alpha):
    torch, A, O = env
    pts_h = c1.points[:n]
    ds = O.Dataset(pts_h, 0)
    say(f"clustering-based build n={n} T={T} Ls={Ls} s={s} l={l} R={R}")
    og = O.hcnng_build(ds, T, Ls, s, l, R, alpha, seed=7, threads=0)
    pts = dev(torch, pts_h)
    g = A.ann_hcnng_build(pts, T, Ls, s, l, R, alpha, seed=7)
    rows = g.neighbors()
    bad = np.nonzero((rows != og).any(1))[0]
    assert len(bad) == 0, f"rows differ: {bad[:10]}"
    assert g.info().start == O.start_vertex(ds)
    # the flat graph's search serves it
    ids, dists = A.ann_search(g, pts, dev(torch, c1.queries), 10, 40)
    oi, od = O.search_batch(ds, og, O.start_vertex(ds), c1.queries, 10, 40, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # deterministic
    assert (A.ann_hcnng_build(pts, T, Ls, s, l, R, alpha, seed=7).neighbors() == rows).all()


def test_hcnng_int8_padded_rows(env):
    torch, A, O = env
    w = W.c3(n=4000, nq=200)
    ds = O.Dataset(w.points, 0)
    og = O.hcnng_build(ds, 8, 100, 3, 10, 24, 1.2, seed=3, threads=0)
    g = A.ann_hcnng_build(dev(torch, w.points), 8, 100, 3, 10, 24, 1.2, seed=3)
    assert (g.neighbors() == og).all()


def test_hcnng_bad_arguments(env, c1):
    torch, A, O = env
    pts = dev(torch, c1.points[:500])
    ok = dict(T=4, Ls=100, s=3, l=10, R=16, alpha=1.2)
    for bad in (dict(T=0), dict(Ls=1), dict(Ls=2000), dict(s=0), dict(s=300), dict(l=0), dict(l=17), dict(R=0),
                dict(alpha=0.0)):
        with pytest.raises(A.AnnError):
            say(f"  refused: {bad}")
            A.ann_hcnng_build(pts, **{**ok, **bad})
    with pytest.raises(A.AnnError):  # float rows above 1,024 bytes are not taken
        A.ann_hcnng_build(dev(torch, np.zeros((100, 260), np.float32)), **ok)
    with pytest.raises(A.AnnError):  # the inner product is for float data
        A.ann_hcnng_build(pts, metric=A.MIPS, **ok)
    with pytest.raises(A.AnnError):  # rows above 128 bytes neither
        A.ann_hcnng_build(dev(torch, np.zeros((100, 256), np.uint8)), **ok)


def test_hcnng_c2_full_size(env):
    """At the benchmark's size (a million 128-byte points, leaves of up to 1,000, s = 3, l = 10):
    two cluster trees against the oracle's in full; the accepted pairs of sampled leaves against
    the oracle's; and the rows of a four-tree build, for sampled points, against the oracle's
    prune of the neighbours that the four trees give."""
    torch, A, O = env
    w = W.c2()
    ds = O.Dataset(w.points, 0)
    pts = dev(torch, w.points)
    T, Ls, s, l, R, alpha, seed = 4, 1000, 3, 10, 64, 1.2, 9
    rng = np.random.default_rng(0)
    nb_u, nb_v = [], []
    for t in range(T):
        perm, off, pairs = A.ann_hcnng_tree_edges(pts, Ls, s, l, seed, t)
        nb_u.append(pairs[:, 0])
        nb_v.append(pairs[:, 1])
        if t in (0, 3):
            say(f"tree {t}: {len(off) - 1} leaves, {len(pairs)} pairs; oracle cuts the same tree")
            operm, ooff = O.hcnng_tree(ds, Ls, seed, t)
            assert (off == ooff).all() and (perm == operm).all()
            leaf_of = np.empty(w.n, np.int64)
            leaf_of[perm] = np.repeat(np.arange(len(off) - 1), np.diff(off))
            pl = leaf_of[pairs[:, 0]]
            assert (pl == leaf_of[pairs[:, 1]]).all() and (np.diff(pl) >= 0).all()
            for j in rng.choice(len(off) - 1, 12, replace=False):
                want = O.hcnng_leaf(ds, perm[off[j]:off[j + 1]], s, l)
                assert (pairs[pl == j] == want).all(), f"tree {t} leaf {j}"
    u = np.concatenate(nb_u + nb_v).astype(np.int64)
    v = np.concatenate(nb_v + nb_u).astype(np.int64)
    order = np.lexsort((v, u))
    u, v = u[order], v[order]
    keep = np.ones(len(u), bool)
    keep[1:] = (u[1:] != u[:-1]) | (v[1:] != v[:-1])
    u, v = u[keep], v[keep]
    first = np.searchsorted(u, np.arange(w.n + 1))
    say("four-tree build")
    g = A.ann_hcnng_build(pts, T, Ls, s, l, R, alpha, seed=seed)
    rows = g.neighbors()
    deg = (rows != NONE).sum(1)
    assert deg.max() <= R and (deg > 0).mean() > 0.999
    for p in rng.choice(w.n, 2000, replace=False):
        cand = v[first[p]:first[p + 1]].astype(np.uint32)
        assert row_list(rows[p]) == O.prune(ds, w.points[p], int(p), cand, R, alpha).tolist(), f"point {p}"


@pytest.mark.parametrize("metric,alpha", [(0, 1.2), (1, 1.0)])
def test_hcnng_f32(env, metric, alpha):
    """Float data: sums run in fp32 (squared L2 inside a leaf as |a|^2 + |b|^2 - 2<a,b> on the
    fp32 matrix cores), so near-ties may fall the other way than in the oracle's fp64 sums and
    move a point to the other side of a cut, or swap a neighbour or a tree edge.  Bounded here:
    nearly every point in the same leaf, nearly every pair and row the same, recall within 0.002."""
    torch, A, O = env
    w = W.c4(n=6000, nq=400)
    ds = O.Dataset(w.points, metric)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    Ls, s, l = 150, 3, 10
    perm, off, pairs = A.ann_hcnng_tree_edges(pts, Ls, s, l, 3, 1, metric=metric)
    operm, ooff, opairs = _oracle_tree_pairs(O, ds, Ls, s, l, 3, 1)
    assert sorted(perm.tolist()) == list(range(w.n)) and (np.diff(off) <= Ls).all() and (np.diff(off) >= 1).all()

    def leaf_ids(perm, off):
        sig = np.empty(w.n, np.int64)
        for j in range(len(off) - 1):
            ids = perm[off[j]:off[j + 1]]
            assert (np.diff(ids.astype(np.int64)) > 0).all()
            sig[ids] = int(ids[0]) * 100000 + len(ids)
        return sig
    same_leaf = (leaf_ids(perm, off) == leaf_ids(operm, ooff)).mean()
    got = {(int(a), int(b)) for a, b in pairs}
    want = {(int(a), int(b)) for a, b in opairs}
    say(f"  metric {metric}: same leaf {same_leaf:.4f}, pairs in common {len(got & want) / len(want):.4f}")
    assert same_leaf > 0.98 and len(got & want) / len(want) > 0.97
    deg = np.bincount(pairs.ravel(), minlength=w.n)
    assert deg.max() <= s

    T, R = 8, 32
    og = O.hcnng_build(ds, T, Ls, s, l, R, alpha, seed=3, threads=0)
    g = A.ann_hcnng_build(pts, T, Ls, s, l, R, alpha, seed=3, metric=metric)
    rows = g.neighbors()
    same_rows = (rows == og).all(1).mean()
    say(f"  rows identical {same_rows:.4f}")
    assert same_rows >= 0.99
    gt, _ = O.brute_force(ds, w.queries, 10)
    st = O.start_vertex(ds)
    assert g.info().start == st
    gi, _ = A.ann_search(g, pts, qs, 10, 64)
    oi, _ = O.search_batch(ds, og, st, w.queries, 10, 64, threads=0)
    r_g, r_o = recall_at_k(gi.cpu().numpy().view(np.uint32), gt), recall_at_k(oi, gt)
    say(f"  recall gpu={r_g:.4f} oracle={r_o:.4f}")
    assert abs(r_g - r_o) <= 0.002


def test_hcnng_single_leaf_and_large_parameters(env, c1):
    torch, A, O = env
    # fewer points than a leaf holds: every tree is one leaf, all trees give the same edges
    for n in (1, 2, 40):
        pts_h = c1.points[:n]
        og = O.hcnng_build(O.Dataset(pts_h, 0), 3, 64, 3, 10, 8, 1.2, seed=1)
        assert (A.ann_hcnng_build(dev(torch, pts_h), 3, 64, 3, 10, 8, 1.2, seed=1).neighbors() == og).all()
    # the largest leaf, l and degree bound the library takes
    pts_h = c1.points[:2500]
    og = O.hcnng_build(O.Dataset(pts_h, 0), 2, 1024, 255, 16, 512, 1.5, seed=2, threads=0)
    assert (A.ann_hcnng_build(dev(torch, pts_h), 2, 1024, 255, 16, 512, 1.5, seed=2).neighbors() == og).all()


def test_hnsw_wide_layers(env, c1):
    """m = 128 (bottom rows of 256 ids, four beam slots at efc = 300)."""
    torch, A, O = env
    n = 2500
    ds = O.Dataset(c1.points[:n], 0)
    oh = O.hnsw_build(ds, 128, 300, 1.2, seed=6, level=(np.arange(n) % 7 == 0).astype(np.uint32), threads=0)
    pts = dev(torch, c1.points[:n])
    h = A.ann_hnsw_build(pts, 128, 300, 1.2, seed=6, level=(np.arange(n) % 7 == 0).astype(np.uint32))
    _check_hnsw_against(h, oh, n)
    ids, dists = A.ann_hnsw_search(h, pts, dev(torch, c1.queries), 10, 300)
    oi, od, _ = O.hnsw_search_batch(ds, oh, c1.queries, 10, 300, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()


def test_hnsw_insert_points(env, c1):
    """Points streamed into the layered index: every layer identical to the oracle's after each
    call; levels by the index's rule, capped; a build cut at a batch boundary and continued this
    way is the one-shot build."""
    torch, A, O = env
    m, efc, alpha = 8, 40, 1.2
    cuts = (5000, 7000, c1.n)
    pts, qs = dev(torch, c1.points), dev(torch, c1.queries)
    oh = O.hnsw_build(O.Dataset(c1.points[:cuts[0]], 0), m, efc, alpha, seed=5, threads=0)
    h = A.ann_hnsw_build(pts[:cuts[0]], m, efc, alpha, seed=5)
    _check_hnsw_against(h, oh, cuts[0])
    for seed, n_tot in ((3, cuts[1]), (4, cuts[2])):
        say(f"layered index: points up to {n_tot}")
        ds = O.Dataset(c1.points[:n_tot], 0)
        oh = O.hnsw_insert_points(ds, oh, efc, alpha, seed=seed, level_seed=5, threads=0)
        A.ann_hnsw_insert_points(h, pts[:n_tot], efc, alpha, seed=seed)
        assert h.info().n == n_tot
        _check_hnsw_against(h, oh, n_tot)
        ids, dists = A.ann_hnsw_search(h, pts[:n_tot], qs, 10, 40)
        oi, od, _ = O.hnsw_search_batch(ds, oh, c1.queries, 10, 40, threads=0)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # continuation of a build
    n, theta = 4000, 250
    rng = np.random.default_rng(3)
    level = np.minimum(rng.geometric(0.7, n) - 1, 3).astype(np.uint32)
    level[0] = 3
    order = np.arange(1, n, dtype=np.uint32)
    whole = A.ann_hnsw_build(pts[:n], m, efc, alpha, batch_cap=theta, level=level, order=order)
    b = O.schedule(n - 1, theta).astype(np.int64)
    n1 = int(b[10]) + 1
    part = A.ann_hnsw_build(pts[:n1], m, efc, alpha, batch_cap=theta, level=level[:n1], order=order[:n1 - 1])
    A.ann_hnsw_insert_points(part, pts[:n], efc, alpha, batch_cap=theta, order=order[n1 - 1:], level=level[n1:])
    for l in range(4):
        (ia, ra), (ib, rb) = whole.layer(l), part.layer(l)
        assert (ia == ib).all() and (ra == rb).all()
    # refused calls
    with pytest.raises(A.AnnError):
        A.ann_hnsw_insert_points(part, pts[:100], efc, alpha)
    with pytest.raises(A.AnnError):
        A.ann_hnsw_insert_points(part, pts[:n + 10], efc, alpha, order=np.arange(10, dtype=np.uint32))


def test_hnsw_insert_points_padded_rows(env):
    torch, A, O = env
    w = W.c3(n=5000, nq=200)
    oh = O.hnsw_build(O.Dataset(w.points[:3000], 0), 10, 40, 1.0, seed=2, threads=0)
    pts = dev(torch, w.points)
    h = A.ann_hnsw_build(pts[:3000], 10, 40, 1.0, seed=2)
    ds = O.Dataset(w.points, 0)
    oh = O.hnsw_insert_points(ds, oh, 40, 1.0, seed=8, level_seed=2, threads=0)
    A.ann_hnsw_insert_points(h, pts, 40, 1.0, seed=8)
    _check_hnsw_against(h, oh, w.n)
    ids, dists = A.ann_hnsw_search(h, pts, dev(torch, w.queries), 10, 50)
    oi, od, _ = O.hnsw_search_batch(ds, oh, w.queries, 10, 50, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
