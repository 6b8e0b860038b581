"""Pins for the oracle's prune(p, C, R) (Sec. 4.1)."""
import json
import os

import numpy as np
import pytest

from helpers import audit_prune, exact_knn

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_cases(oracle):
    f = json.load(open(os.path.join(GOLD, "prune_1d.json")))
    pts = np.array(f["points"], np.int8)
    ds = oracle.Dataset(pts, 0)
    p = f["p"]
    for case in f["cases"]:
        out = oracle.prune(ds, pts[p], p, np.array(case["cand"]), case["R"], case["alpha"])
        assert out.tolist() == case["expect"], case["derivation"]


def _rand(rng, n, d, dtype):
    if dtype == np.uint8:
        return rng.integers(0, 256, (n, d)).astype(np.uint8)
    if dtype == np.int8:
        return rng.integers(-127, 128, (n, d)).astype(np.int8)
    x = rng.standard_normal((n, d))
    return (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)


@pytest.mark.parametrize("dtype", [np.uint8, np.int8, np.float32])
def test_huge_alpha_keeps_the_R_closest(oracle, dtype):
    """alpha so large that nothing is dominated (no duplicate vectors): the result is the
    first R candidates in (distance, id) order."""
    rng = np.random.default_rng(1)
    pts = _rand(rng, 80, 6, dtype)
    ds = oracle.Dataset(pts, 0)
    for _ in range(10):
        cand = rng.choice(np.arange(1, 80), size=30, replace=False)
        out = oracle.prune(ds, pts[0], 0, cand, 8, 1e9)
        e, _ = exact_knn(pts, pts[0], 8, 0, subset=cand.tolist())
        assert out.tolist() == e.tolist()


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_tiny_alpha_keeps_only_the_closest(oracle, dtype):
    rng = np.random.default_rng(2)
    pts = _rand(rng, 80, 6, dtype)
    ds = oracle.Dataset(pts, 0)
    for _ in range(10):
        cand = rng.choice(np.arange(1, 80), size=30, replace=False)
        out = oracle.prune(ds, pts[0], 0, cand, 8, 1e-9 if dtype == np.float32 else 0.0)
        e, _ = exact_knn(pts, pts[0], 1, 0, subset=cand.tolist())
        assert out.tolist() == e.tolist()


@pytest.mark.parametrize("dtype,metric,alpha", [
    (np.uint8, 0, 1.2), (np.int8, 0, 1.2), (np.uint8, 0, 1.0), (np.float32, 0, 1.2),
    (np.float32, 1, 1.0), (np.float32, 1, 0.9)])
def test_audit_random(oracle, dtype, metric, alpha):
    """Every kept and every dropped candidate is explained by the rule, checked with
    numpy distances and without re-running the scan."""
    rng = np.random.default_rng(4)
    n, d = 120, 3  # low dimension so that domination actually happens
    pts = _rand(rng, n, d, dtype)
    pts[17] = pts[5]
    ds = oracle.Dataset(pts, metric)
    sizes = []
    for trial in range(25):
        p = int(rng.integers(n))
        m = int(rng.integers(1, 60))
        cand = rng.integers(0, n, size=m)  # may repeat and may contain p
        R = int(rng.integers(1, 12))
        st = oracle.Stats()
        out = oracle.prune(ds, pts[p], p, cand, R, alpha, stats=st)
        audit_prune(pts, pts[p], p, cand, out, R, alpha, metric)
        sizes.append(len(out))
    assert min(sizes) >= 1 and len(set(sizes)) > 2


def test_empty_and_self_only(oracle):
    pts = np.zeros((3, 4), np.uint8)
    ds = oracle.Dataset(pts, 0)
    assert oracle.prune(ds, pts[0], 0, np.array([], np.uint32), 4, 1.2).tolist() == []
    assert oracle.prune(ds, pts[0], 0, np.array([0, 0]), 4, 1.2).tolist() == []
    # duplicates of the same vector: the first dominates the second (alpha*0 <= d)
    assert oracle.prune(ds, pts[0], 0, np.array([2, 1]), 4, 1.2).tolist() == [1]
