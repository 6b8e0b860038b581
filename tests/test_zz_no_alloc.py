"""ann_search_noalloc, the query search that allocates nothing, against ann_search / ann_search_eps
through the C ABI: same ids and distances, bit for bit, on two calls in a row, the second with
fewer queries (the staging array keeps the first call's contents)."""
import numpy as np
import pytest

from helpers import dev
from paper_2305_04359_amd import workloads as W

pytestmark = pytest.mark.gpu


def _outputs(torch, nq, k, f32=False):
    ids = torch.full((nq, k), -7, dtype=torch.int32, device="cuda:0")
    dists = torch.full((nq, k), -7, dtype=torch.float32 if f32 else torch.int32, device="cuda:0")
    return ids, dists


def test_search_noalloc_matches_search(env):
    torch, A, O = env
    # int8 rows of 100 bytes: the queries are staged, zero-padded to 128 bytes, in the library's array
    w = W.c3(n=5000, nq=700)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    g = A.ann_build(pts, 24, 48, 1.2, seed=2)
    og, s = O.build(O.Dataset(w.points, 0), 24, 48, 1.2, seed=2, threads=0)
    assert (g.neighbors() == og).all()
    k = 10
    for nq, L, eps in ((700, 60, -1.0), (130, 35, -1.0), (700, 40, 0.1), (1, 20, -1.0), (333, 600, -1.0)):
        want_i, want_d = A.ann_search(g, pts, qs[:nq], k, L, eps=None if eps < 0 else eps)
        ids, dists = _outputs(torch, nq, k)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        A.ann_search_noalloc(g, pts, qs[:nq], k, L, ids, dists, eps=eps)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert (ids == want_i).all() and (dists == want_d).all(), f"nq={nq} L={L} eps={eps}"
        oi, od = O.search_batch(O.Dataset(w.points, 0), og, s, w.queries[:nq], k, L, threads=0, eps=eps)
        assert (ids.cpu().numpy().view(np.uint32) == oi).all() and (dists.cpu().numpy() == od).all()
    # more queries than the array can stage: refused, outputs untouched
    many = torch.zeros((65537, 100), dtype=torch.int8, device="cuda:0")
    ids, dists = _outputs(torch, 65537, 1)
    with pytest.raises(A.AnnError) as e:
        A.ann_search_noalloc(g, pts, many, 1, 8, ids, dists)
    assert e.value.code == -1 and "65536" in str(e.value)
    assert (ids == -7).all()
    A.ann_search_noalloc(g, pts, many[:65536], 1, 8, ids[:65536], dists[:65536])  # the largest that fits
    torch.cuda.synchronize()
    assert (ids[:65536] >= 0).all()
    # a graph that has not seen this points array yet holds no padded copy of it
    gh = A.ann_graph_from_host(og, w.d, A.I8, A.L2SQ, s)
    ids, dists = _outputs(torch, 50, k)
    with pytest.raises(A.AnnError):
        A.ann_search_noalloc(gh, pts, qs[:50], k, 30, ids, dists)
    want_i, want_d = A.ann_search(gh, pts, qs[:50], k, 30)  # makes the copy
    A.ann_search_noalloc(gh, pts, qs[:50], k, 30, ids, dists)
    assert (ids == want_i).all() and (dists == want_d).all()


def test_search_noalloc_rows_that_need_no_staging(env):
    torch, A, O = env
    w = W.c1(n=3000, nq=400)
    pts, qs = dev(torch, w.points), dev(torch, w.queries)
    g = A.ann_build(pts, 16, 32, 1.2, seed=1)
    for nq in (400, 77):
        want_i, want_d = A.ann_search(g, pts, qs[:nq], 10, 50)
        ids, dists = _outputs(torch, nq, 10)
        A.ann_search_noalloc(g, pts, qs[:nq], 10, 50, ids, dists)
        assert (ids == want_i).all() and (dists == want_d).all()
    wf = W.c4(n=2000, nq=100)
    pf, qf = dev(torch, wf.points), dev(torch, wf.queries)
    gf = A.ann_build(pf, 16, 32, 1.0, seed=1, metric=A.MIPS)
    want_i, want_d = A.ann_search(gf, pf, qf, 10, 40)
    ids, dists = _outputs(torch, 100, 10, f32=True)
    A.ann_search_noalloc(gf, pf, qf, 10, 40, ids, dists)
    assert (ids == want_i).all() and (dists == want_d).all()
