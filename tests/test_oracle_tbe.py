"""Pins for the oracle's thought-adaptive eviction: K-means survivor choice and the annealing plan (CPU only)."""
import numpy as np
import pytest

from oracle import cache as oc
from oracle import tbe


def test_one_dimensional_example_by_hand():
    # two groups on a line; K = 2, initial centroids are points 0 and 3
    x = np.array([[0.0], [1.0], [2.0], [10.0], [11.0], [12.5]])
    keep, margin, obj = tbe.kmeans_select(x, 2)
    # assignment {0,1,2} / {3,4,5}; means 1 and 11.1666...; nearest members: 1 and 11
    assert keep.tolist() == [1, 4]
    assert obj[0] == pytest.approx(1 + 4 + 0 + 1 + 2.5 ** 2) and obj[-1] == pytest.approx(2.0 + (1.1666666666666667 ** 2 + 0.16666666666666666 ** 2 + 1.3333333333333333 ** 2))
    assert margin > 0.01


def test_everything_survives_when_keep_covers_the_segment():
    x = np.random.default_rng(0).standard_normal((5, 8))
    for keep in (5, 6, 64):
        s, margin, _ = tbe.kmeans_select(x, keep)
        assert s.tolist() == [0, 1, 2, 3, 4] and margin == np.inf


def test_separated_blobs_one_survivor_each_nearest_the_blob_mean():
    rng = np.random.default_rng(1)
    K, per, dim = 8, 12, 32
    centres = rng.standard_normal((K, dim)) * 50
    # blob b owns points b * per .. (b + 1) * per - 1, so the evenly spaced initial centroids fall one
    # into each blob (Lloyd is a local search: from such a start it has to end on the blobs)
    blob = np.arange(K * per) // per
    x = centres[blob] + rng.standard_normal((K * per, dim))
    keep, margin, obj = tbe.kmeans_select(x, K, max_iters=20)
    assert len(keep) == K and sorted(blob[keep].tolist()) == list(range(K))
    for b in range(K):
        members = np.flatnonzero(blob == b)
        mean = x[members].mean(axis=0)
        nearest = members[np.argmin(((x[members] - mean) ** 2).sum(axis=1))]
        assert nearest in keep
    assert all(b <= a + 1e-9 for a, b in zip(obj, obj[1:]))          # Lloyd never increases the objective


def test_same_partition_as_the_library_lloyd_from_the_same_start():
    sk = pytest.importorskip("sklearn.cluster")
    rng = np.random.default_rng(2)
    n, k, dim = 150, 16, 24
    x = rng.standard_normal((n, dim)) + rng.integers(0, 6, size=(n, 1)) * 3.0
    init = x[(np.arange(k) * n) // k]
    km = sk.KMeans(n_clusters=k, init=init, n_init=1, algorithm="lloyd", max_iter=300, tol=0.0).fit(x)
    keep, margin, obj = tbe.kmeans_select(x, k, max_iters=300)
    assert margin > 1e-9
    assert obj[-1] == pytest.approx(km.inertia_, rel=1e-9)
    # survivors = per library cluster the member nearest the library centroid
    want = []
    for j in range(k):
        members = np.flatnonzero(km.labels_ == j)
        if len(members) <= 2:
            want.append(int(members[0]))
        else:
            want.append(int(members[np.argmin(((x[members] - km.cluster_centers_[j]) ** 2).sum(axis=1))]))
    assert sorted(want) == keep.tolist()


def test_ties_and_empty_clusters():
    # duplicates: points 0 and 1 coincide, so do 2 and 3; K = 3 starts at points 0, 1, 2 -> cluster 1 never gets a point
    x = np.array([[0.0, 0.0], [0.0, 0.0], [5.0, 5.0], [5.0, 5.0]])
    keep, margin, _ = tbe.kmeans_select(x, 3)
    assert keep.tolist() == [0, 2] and margin == 0.0            # ties go to the lowest cluster / index; two survivors only
    # iteration cap: a single assignment pass still yields one survivor per non-empty cluster
    rng = np.random.default_rng(3)
    x = rng.standard_normal((40, 6))
    keep, _, obj = tbe.kmeans_select(x, 8, max_iters=1)
    assert len(obj) == 1 and 1 <= len(keep) <= 8


def test_select_evictions_reads_the_stored_keys():
    cfg = oc.OracleConfig(1, 8, 2, 64, (8, 2, 4), 2, 64, (64, 64, 64))
    c = oc.OracleCache(cfg)
    rng = np.random.default_rng(4)
    n = 48
    k = rng.standard_normal((n, 2, 64)).astype(np.float16).astype(np.float32)
    cls = np.repeat(np.array([2, 1, 0], np.uint8), 16)
    h = c.append(0, k, k, np.ones(n, np.int64), np.arange(n), cls)
    off = [0, 16, 32, 48]
    ev, margins = tbe.select_evictions(c, 0, np.ones(n, np.int64), h, off, [4, 8, 16])
    assert margins.shape == (3,) and margins[2] == np.inf          # keep >= size: no decision was taken
    for s, keep in enumerate([4, 8, 16]):
        seg = ev[off[s]:off[s + 1]]
        assert (seg == -1).sum() == min(keep, 16)
        assert np.array_equal(seg[seg != -1], np.asarray(h)[off[s]:off[s + 1]][seg != -1])
    # the clustering sees the dequantised keys: a direct call on them gives the same survivors
    x = tbe.segment_keys(c, 0, 1, h[:16])
    assert x.shape == (16, 128)
    direct, _, _ = tbe.kmeans_select(x, 4)
    assert np.array_equal(np.flatnonzero(ev[:16] == -1), direct)


def test_anneal_plan_cases():
    T, E, R = 0, 1, 2
    # Case 1: a transition segment has just ended -> every earlier segment goes down one level; the open segment is left alone
    types = [R, E, T, R]
    cuts = tbe.anneal_plan(types, [128, 100, 40, 10], True, 278, 10 ** 9)
    assert cuts == [(0, 64), (1, 64), (2, 32)]
    # a second transition: next level each; a segment at the floor stays
    cuts = tbe.anneal_plan([R, E, T, R, T, E], [64, 64, 32, 4, 20, 7], True, 191, 10 ** 9)
    assert cuts == [(0, 32), (1, 32), (2, 16), (4, 16)]
    # Case 2: over budget, no transition: least important type first (T, then E, then R), oldest first, one level at a time
    cuts = tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 400)
    assert cuts == [(2, 64), (2, 32), (2, 16)] or cuts[:1] == [(2, 64)]
    total = 562
    live = [128, 128, 128, 128, 50]
    for i, r in cuts:
        total -= live[i] - r
        live[i] = r
    assert total <= 400 and live[4] == 50
    # nothing can shrink any more: the plan stops even though the budget is not met
    assert tbe.anneal_plan([T, T, R], [4, 4, 500], False, 508, 100) == []


def test_anneal_plan_one_cut_per_segment_and_capacity():
    T, E, R = 0, 1, 2
    # over budget by a lot: with once=True the transition segment is cut once, then the plan moves on to the next candidates
    cuts = tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 300, once=True)
    assert cuts == [(2, 64), (1, 64), (3, 64), (0, 64)]
    # capacity: stops after max_cuts cuts
    assert tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 300, once=True, max_cuts=2) == [(2, 64), (1, 64)]
    # Case 1 and Case 2 in one call: the transition cut is not repeated by Case 2
    cuts = tbe.anneal_plan([T, R, T, E], [100, 100, 20, 9], True, 229, 60, once=True)
    assert cuts == [(0, 64), (1, 64), (2, 16)]


def test_plan_evictions_groups_live_tokens_by_segment_start():
    cfg = oc.OracleConfig(1, 8, 2, 64, (8, 2, 4), 1, 64, (64, 64, 64))
    c = oc.OracleCache(cfg)
    rng = np.random.default_rng(5)
    n = 300
    types = np.array([2] * 100 + [0] * 80 + [1] * 120, np.uint8)          # three segments: R, T, E (the last one open)
    k = rng.standard_normal((n, 2, 64)).astype(np.float16).astype(np.float32)
    h = np.asarray(c.append(0, k, k, np.zeros(n, np.int64), np.arange(n), types))
    c.evict_slots(0, [0] * 10, h[5:15])                                    # ten tokens of segment 0 are gone already
    plan = tbe.plan_evictions(c, 0, 0, [0, 100, 180], [2, 0, 1], True, 10 ** 9, 8)
    assert [(i, r) for i, r, _ in plan] == [(0, 64), (1, 64)]
    assert plan[0][2] == [int(x) for x in np.r_[h[:5], h[15:100]]]         # live tokens of the segment, ascending position
    assert plan[1][2] == [int(x) for x in h[100:180]]
    # no trigger, within budget: nothing
    assert tbe.plan_evictions(c, 0, 0, [0, 100, 180], [2, 0, 1], False, 290, 8) == []
    # over budget: the transition segment first (least important), then execution is open, so reasoning
    plan = tbe.plan_evictions(c, 0, 0, [0, 100, 180], [2, 0, 1], False, 200, 8)
    assert [(i, r) for i, r, _ in plan] == [(1, 64), (0, 64)]
