"""Independent numpy re-statements used to pin the oracle (never the oracle's own code)."""
from __future__ import annotations

import numpy as np

NONE = 0xFFFFFFFF


def np_dist(a, b, metric=0):
    """Exact distance for integer vectors (python ints), float64 for floats."""
    if a.dtype in (np.uint8, np.int8):
        x = a.astype(np.int64)
        y = b.astype(np.int64)
        return int(((x - y) ** 2).sum()) if metric == 0 else int(-(x * y).sum())
    x = a.astype(np.float64)
    y = b.astype(np.float64)
    v = ((x - y) ** 2).sum() if metric == 0 else -(x * y).sum()
    return float(np.float32(v) + np.float32(0.0))


def np_dists_to(points, q, metric=0):
    if points.dtype in (np.uint8, np.int8):
        x = points.astype(np.int64)
        y = q.astype(np.int64)[None, :]
        return ((x - y) ** 2).sum(1) if metric == 0 else -(x * y).sum(1)
    x = points.astype(np.float64)
    y = q.astype(np.float64)[None, :]
    v = ((x - y) ** 2).sum(1) if metric == 0 else -(x * y).sum(1)
    return v.astype(np.float32).astype(np.float64) + 0.0


def exact_knn(points, q, k, metric=0, subset=None):
    """k nearest under (distance, id), by full sort."""
    ids = np.arange(points.shape[0]) if subset is None else np.asarray(sorted(subset))
    d = np_dists_to(points[ids], q, metric)
    order = np.lexsort((ids, d))[:k]
    return ids[order].astype(np.uint32), d[order]


def alpha_dominates(dtype, alpha, d_star_c, d_p_c):
    if dtype in (np.uint8, np.int8):
        a16 = int(round(alpha * 65536.0))
        return a16 * int(d_star_c) <= int(d_p_c) * 65536
    return bool(np.float32(alpha) * np.float32(d_star_c) <= np.float32(d_p_c))


def audit_prune(points, p_vec, p_id, cand, out, R, alpha, metric=0):
    """Check a prune result against the rule of Sec. 4.1 without re-running the scan:
    kept points are in (dist,id) order; no kept point is dominated by an earlier kept point;
    every dropped point is dominated by a kept point that precedes it, or was cut by |out| = R."""
    dt = points.dtype
    cset = sorted({int(c) for c in cand if int(c) != NONE and int(c) != p_id})
    out = [int(x) for x in out]
    assert len(out) <= R
    assert len(set(out)) == len(out)
    assert all(o in cset for o in out)
    if cset:
        assert len(out) >= 1
    key = {c: (np_dist(p_vec, points[c], metric), c) for c in cset}
    assert [key[o] for o in out] == sorted(key[o] for o in out)
    for i, x in enumerate(out):
        for y in out[:i]:
            assert not alpha_dominates(dt, alpha, np_dist(points[y], points[x], metric), key[x][0]), \
                f"kept {x} is dominated by earlier kept {y}"
    kept = set(out)
    for c in cset:
        if c in kept:
            continue
        dominated = any(
            key[y] < key[c] and alpha_dominates(dt, alpha, np_dist(points[y], points[c], metric), key[c][0])
            for y in out)
        cut = len(out) == R and key[c] > key[out[-1]]
        assert dominated or cut, f"dropped {c} without reason"


def recall_at_k(ids, gt):
    k = gt.shape[1]
    return float(np.mean([len(set(a.tolist()) & set(b.tolist())) / k for a, b in zip(ids, gt)]))


def row_list(row):
    return [int(x) for x in row if int(x) != NONE]


def dev(torch, a):
    """A host array as a device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def say(msg):
    print(msg, flush=True)
