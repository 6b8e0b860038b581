"""GPU tests of the boundary itself: wide beams, the allocator callbacks, argument checks that
need the device, and the counters' switch.  All results are compared with the CPU oracle."""
import numpy as np
import pytest

from helpers import dev, say
from paper_2305_04359_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c1():
    return W.c1()


@pytest.fixture(scope="module")
def c1_oracle(oracle, c1):
    ds = oracle.Dataset(c1.points, 0)
    g, s = oracle.build(ds, c1.R, c1.L, c1.alpha, seed=c1.seed, threads=0)
    return ds, g, s


@pytest.mark.parametrize("L,k", [(513, 10), (600, 10), (1000, 100), (1024, 1000), (1025, 10), (2048, 70)])
def test_search_wide_beams_bit_exact(env, c1, c1_oracle, L, k):
    """Beams beyond 512 entries (Sec. 4.5 sweeps the beam width to reach high recall): 16 and 32
    beam slots per lane, with and without the (1 + eps) rule."""
    torch, A, O = env
    ds, og, s = c1_oracle
    pts = dev(torch, c1.points)
    g = A.ann_graph_from_host(og, c1.d, A.U8, A.L2SQ, s)
    qs_h = c1.queries[:200]
    qs = dev(torch, qs_h)
    for eps in (None, 0.1):
        ids, dists = A.ann_search(g, pts, qs, k, L, eps=eps)
        oi, od = O.search_batch(ds, og, s, qs_h, k, L, threads=0, eps=-1.0 if eps is None else eps)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all(), f"ids differ at L={L} eps={eps}"
        assert (dists.cpu().numpy() == od).all(), f"distances differ at L={L} eps={eps}"


def test_search_wide_beams_other_types_and_limits(env):
    torch, A, O = env
    # float rows, inner product, a beam wider than the graph has vertices
    w = W.c4(n=1500, nq=60)
    ds = O.Dataset(w.points, 1)
    og, s = O.build(ds, 16, 32, 1.0, seed=1, threads=0)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    g = A.ann_graph_from_host(og, w.d, A.F32, A.MIPS, s)
    ids, dists = A.ann_search(g, pts, qs, 10, 2048)
    oi, od = O.search_batch(ds, og, s, w.queries, 10, 2048, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).mean() >= 0.99  # fp32 near-ties
    assert np.allclose(dists.cpu().numpy(), od, rtol=1e-5, atol=1e-6)
    # int8 rows of 100 bytes (padded inside the library), beam 700
    w3 = W.c3(n=3000, nq=80)
    ds3 = O.Dataset(w3.points, 0)
    og3, s3 = O.build(ds3, 16, 32, 1.2, seed=1, threads=0)
    p3 = dev(torch, w3.points)
    g3 = A.ann_graph_from_host(og3, w3.d, A.I8, A.L2SQ, s3)
    ids, dists = A.ann_search(g3, p3, dev(torch, w3.queries), 10, 700)
    oi, od = O.search_batch(ds3, og3, s3, w3.queries, 10, 700, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # the layered index takes the same beams
    oh = O.hnsw_build(ds3, 8, 32, 1.2, seed=2, threads=0)
    h = A.ann_hnsw_build(p3, 8, 32, 1.2, seed=2)
    ids, dists = A.ann_hnsw_search(h, p3, dev(torch, w3.queries), 10, 900)
    oi, od, _ = O.hnsw_search_batch(ds3, oh, w3.queries, 10, 900, threads=0)
    assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    with pytest.raises(A.AnnError):
        A.ann_search(g3, p3, dev(torch, w3.queries), 10, 2049)
    with pytest.raises(A.AnnError):
        A.ann_build(p3, 16, 513, 1.2)  # builds keep the beam at 512


class CountingAllocator:
    """alloc / free callbacks over torch tensors that records every call (and can run dry)."""

    def __init__(self, A, torch, fail_after=None):
        self.A, self.torch = A, torch
        self.live = {}
        self.allocs = self.frees = 0
        self.fail_after = fail_after

        def _alloc(nbytes, stream, user):
            if self.fail_after is not None and self.allocs >= self.fail_after:
                return None
            t = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device="cuda:0")
            p = (t.data_ptr() + 255) // 256 * 256
            self.live[p] = t
            self.allocs += 1
            return p

        def _free(ptr, user):
            del self.live[ptr]
            self.frees += 1

        self.alloc = A.ALLOC_FN(_alloc)
        self.free = A.FREE_FN(_free)

    def fill(self, opts):
        import ctypes as C
        opts.alloc = C.cast(self.alloc, C.c_void_p)
        opts.free = C.cast(self.free, C.c_void_p)
        opts.alloc_user = None


def test_allocator_callbacks(env, c1, c1_oracle):
    """The graph and every scratch buffer come from the caller's callbacks and go back to them;
    the result does not depend on where the memory comes from."""
    torch, A, O = env
    ds, og, s = c1_oracle
    pts = dev(torch, c1.points)
    rows = {}
    for name in (None, "torch"):
        g = A.ann_build(pts, c1.R, c1.L, c1.alpha, seed=c1.seed, allocator=name)
        rows[name] = g.neighbors()
        ids, _ = A.ann_search(g, pts, dev(torch, c1.queries[:50]), 10, 40)
        assert (ids.cpu().numpy().view(np.uint32) == O.search_batch(ds, og, s, c1.queries[:50], 10, 40)[0]).all()
        del g
    assert (rows[None] == og).all() and (rows["torch"] == og).all()
    ca = CountingAllocator(A, torch)
    g = A.ann_build(pts, c1.R, c1.L, c1.alpha, seed=c1.seed, allocator=ca)
    assert (g.neighbors() == og).all()
    say(f"  a build made {ca.allocs} allocations; {len(ca.live)} are the graph's")
    assert ca.allocs >= 10 and len(ca.live) == 3  # rows, degrees, counters stay; all scratch went back
    # insertions after the build draw on the graph's allocator too, and keep their scratch
    g2 = A.ann_build(pts[:8000], c1.R, c1.L, c1.alpha, seed=c1.seed, allocator=ca)
    before = ca.allocs
    A.ann_insert_points(g2, pts, c1.L, c1.alpha, seed=3)
    assert ca.allocs > before
    og2 = O.insert_points(ds, O.build(O.Dataset(c1.points[:8000], 0), c1.R, c1.L, c1.alpha, seed=c1.seed,
                                      threads=0)[0], int(g2.info().start), c1.L, c1.alpha, seed=3, threads=0)
    assert (g2.neighbors() == og2).all()
    del g, g2
    assert len(ca.live) == 0 and ca.allocs == ca.frees
    # the layered index
    h = A.ann_hnsw_build(pts, 8, 32, 1.2, seed=2, allocator=ca)
    oh = O.hnsw_build(ds, 8, 32, 1.2, seed=2, threads=0)
    for l in range(oh.top + 1):
        lid, lrows = h.layer(l)
        assert (lrows == oh.layers[l][lid]).all()
    A.ann_hnsw_search(h, pts, dev(torch, c1.queries[:50]), 10, 40)
    torch.cuda.synchronize()
    del h
    assert len(ca.live) == 0 and ca.allocs == ca.frees
    # an allocator that runs dry part of the way: ANN_ENOMEM, and everything handed out comes back
    for k in (0, 2, 7):
        dry = CountingAllocator(A, torch, fail_after=k)
        with pytest.raises(A.AnnError) as e:
            A.ann_build(pts, c1.R, c1.L, c1.alpha, seed=c1.seed, allocator=dry)
        assert e.value.code == -2
        assert len(dry.live) == 0 and dry.allocs == dry.frees == k
    # one callback without the other
    import ctypes as C
    o = A.BuildOpts()
    o.alloc = C.cast(ca.alloc, C.c_void_p)
    h_out = C.c_void_p()
    rc = A.lib().ann_build(pts.data_ptr(), pts.shape[0], pts.shape[1], A.U8, A.L2SQ, 8, 8, 1.2, 1, C.byref(o),
                           None, C.byref(h_out))
    assert rc == -1 and not h_out.value


def test_insert_batch_checks_its_ids(env, c1):
    torch, A, O = env
    pts = dev(torch, c1.points[:2000])
    g = A.ann_build(pts, 16, 32, 1.2, seed=1, max_rounds=8)  # 182 points and the start vertex are in
    s = int(g.info().start)
    order = O.insertion_order(2000, s, 1)
    rows = g.neighbors()
    new = order[600:700]
    with pytest.raises(A.AnnError):
        A.ann_insert_batch(g, pts, np.concatenate([new, new[:1]]), 32, 1.2)  # an id twice
    with pytest.raises(A.AnnError):
        A.ann_insert_batch(g, pts, np.concatenate([new, order[:1]]), 32, 1.2)  # a point that is in already
    with pytest.raises(A.AnnError):
        A.ann_insert_batch(g, pts, np.array([s], np.uint32), 32, 1.2)
    with pytest.raises(A.AnnError):
        A.ann_insert_batch(g, pts, new, 32, 1e-6)  # rounds to alpha = 0 for integer rows
    assert (g.neighbors() == rows).all()  # nothing was touched
    A.ann_insert_batch(g, pts, new, 32, 1.2)
    og = rows.copy()
    O.batch_insert(O.Dataset(c1.points[:2000], 0), og, s, new, 32, 1.2)
    assert (g.neighbors() == og).all()
    # float rows take any positive alpha
    wf = W.c4(n=600, nq=10)
    gf = A.ann_build(dev(torch, wf.points), 8, 16, 1e-6, seed=1, metric=A.MIPS)
    assert int(gf.info().n) == 600


def test_counters_switch(env, c1, c1_oracle):
    torch, A, O = env
    ds, og, s = c1_oracle
    pts, qs = dev(torch, c1.points), dev(torch, c1.queries[:100])
    g = A.ann_graph_from_host(og, c1.d, A.U8, A.L2SQ, s)
    A.ann_search(g, pts, qs, 10, 40)
    torch.cuda.synchronize()
    assert g.stats()["searches"] == 0
    g.set_stats(True)
    A.ann_search(g, pts, qs, 10, 40)
    torch.cuda.synchronize()
    st = g.stats()
    ost = O.Stats()
    O.search_batch(ds, og, s, c1.queries[:100], 10, 40, stats=ost)
    assert st["searches"] == 100 and st["hops"] == ost.hops and st["evals"] >= ost.evals
    g.set_stats(False)
    A.ann_search(g, pts, qs, 10, 40)
    torch.cuda.synchronize()
    assert g.stats()["searches"] == 100


@pytest.mark.parametrize("kind", ["u8", "f32_l2", "f32_ip", "f32_l2_close"])
def test_hcnng_leaf_neighbours_one_by_one(env, kind):
    """The l nearest neighbours inside a leaf (Sec. 4.3), every (point, neighbour, distance) entry
    checked on its own: integer rows exactly; float rows within 1e-5 of the fp64 value (inner
    products: of sum |p_i q_i|), also where the points of a leaf are a hundredth apart on the unit
    sphere and |a|^2 + |b|^2 - 2<a,b> alone would lose the leading digits."""
    torch, A, O = env
    Ls, l = 150, 10
    if kind == "u8":
        w = W.c1(n=4000, nq=1)
        pts_h, metric = w.points, 0
    elif kind == "f32_l2_close":
        rng = np.random.default_rng(5)
        cen = rng.standard_normal((40, 96))
        cen /= np.linalg.norm(cen, axis=1, keepdims=True)
        x = cen[rng.integers(0, 40, 4000)] + 0.001 * rng.standard_normal((4000, 96))
        pts_h, metric = (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32), 0
    else:
        w = W.c4(n=4000, nq=1)
        pts_h, metric = w.points, (0 if kind == "f32_l2" else 1)
    perm, off, ids, dists = A.ann_hcnng_leaf_knn(dev(torch, pts_h), Ls, l, 3, 1, metric=metric)
    n = len(pts_h)
    assert sorted(perm.tolist()) == list(range(n))
    P = pts_h.astype(np.float64)
    same_lists = 0
    for j in range(len(off) - 1):
        leaf = perm[off[j]:off[j + 1]]
        X = P[leaf]
        if metric == 0:
            D = ((X[:, None, :] - X[None, :, :]) ** 2).sum(-1)
            scale = D
        else:
            D = -(X @ X.T)
            scale = np.abs(X[:, None, :] * X[None, :, :]).sum(-1)
        pos = {int(p): i for i, p in enumerate(leaf)}
        k = min(l, len(leaf) - 1)
        for i, p in enumerate(leaf):
            row_i, row_d = ids[off[j] + i], dists[off[j] + i]
            assert (row_i[k:] == 0xFFFFFFFF).all() and (row_i[:k] != 0xFFFFFFFF).all()
            c = np.array([pos[int(x)] for x in row_i[:k]])
            assert i not in c and len(set(c.tolist())) == k
            ref = D[i, c]
            if pts_h.dtype == np.uint8:
                assert (row_d[:k].astype(np.int64) == ref.astype(np.int64)).all()
            else:
                err = np.abs(row_d[:k].astype(np.float64) - ref)
                assert (err <= 1e-5 * scale[i, c] + 1e-30).all(), \
                    f"leaf {j} point {p}: relative error {np.max(err / (scale[i, c] + 1e-30)):.2e}"
            assert (np.diff(row_d[:k].astype(np.float64)) >= 0).all()
            # the list against the exact one under (distance, position in the leaf)
            d_i = D[i].copy()
            d_i[i] = np.inf
            want = np.lexsort((np.arange(len(leaf)), d_i))[:k]
            same_lists += int((want == c).all())
    share = same_lists / n
    say(f"  {kind}: {len(off) - 1} leaves, lists identical to the exact ones: {share:.4f}")
    assert share == 1.0 if pts_h.dtype == np.uint8 else share >= 0.97


def test_build_with_a_batch_of_a_hundred_thousand_points(env, capsys):
    """Batches of 65,536 and 68,929 points (4.2 and 4.4 million reverse edges): the size at which
    rows with 97 to 512 candidates get a re-prune kernel instance of their own, next to the one
    for hub rows with thousands.  Every row against the oracle."""
    torch, A, O = env
    w = W.c1(n=200_000, nq=10)
    R, L, alpha, cap = 64, 64, 1.2, 140_000
    ds = O.Dataset(w.points, 0)
    og, s = O.build(ds, R, L, alpha, seed=3, theta=cap, threads=0)
    g = A.ann_build(dev(torch, w.points), R, L, alpha, seed=3, batch_cap=cap, collect_stats=True)
    st = g.stats()
    assert g.info().start == s and int(g.info().rounds) == 17
    rows = g.neighbors()
    bad = np.nonzero((rows != og).any(1))[0]
    assert len(bad) == 0, f"{len(bad)} rows differ, first {bad[:10]}"
    with capsys.disabled():
        print(f"\n  [one batch of {cap} points: {st['reprunes']} re-prunes, {st['appends']} appends, graph identical]",
              flush=True)


def test_step_one_in_parts_or_in_one(env):
    """Batches of 8,192 points and more run their searches and prunes in three parts side by side
    on three streams; `step1_parts = 1` keeps them in one.  Same graph either way, the oracle's,
    and the statistics count the launches: with a bound of 9,000 the 30,000-point build has three
    batches of that size after the doubling ones."""
    torch, A, O = env
    w = W.c1(n=30_000, nq=10)
    R, L, alpha, cap = 32, 64, 1.2, 9_000
    ds = O.Dataset(w.points, 0)
    og, s = O.build(ds, R, L, alpha, seed=5, theta=cap, threads=0)
    pts = dev(torch, w.points)
    rows = {}
    for parts in (0, 1):
        g = A.ann_build(pts, R, L, alpha, seed=5, batch_cap=cap, collect_stats=True, step1_parts=parts)
        st = g.stats()
        rounds = int(g.info().rounds)
        big = sum(1 for a, b in zip(O.schedule(w.n - 1, cap)[:-1], O.schedule(w.n - 1, cap)[1:]) if b - a >= 8192)
        assert big >= 2
        assert st["search_launches"] == rounds + (2 * big if parts == 0 else 0)
        assert st["ms_search_launches"] >= st["ms_search"] > 0
        rows[parts] = g.neighbors()
        assert g.info().start == s
    assert (rows[0] == rows[1]).all()
    bad = np.nonzero((rows[0] != og).any(1))[0]
    assert len(bad) == 0, f"{len(bad)} rows differ from the oracle's, first {bad[:10]}"
