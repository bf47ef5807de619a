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


def test_anneal_plan_by_selection_count_hand_made():
    """Problem statement "Thought-Adaptive Eviction" (Sec. 4.3): the n-th selection of a segment keeps min(|segment|, R_n)
    tokens, R = {64, 32, 16, 8, 4}.  Tables worked out by hand."""
    T, E, R = 0, 1, 2
    # Case 1, first transition: every closed segment is selected for the first time (n = 0 -> R_0 = 64).  The 50- and the
    # 40-token segments are smaller than 64: they keep everything (no cut), but their count moves on.  The open segment is left alone.
    cnt = [0, 0, 0, 0, 0]
    cuts = tbe.anneal_plan([R, E, T, E, R], [128, 50, 40, 192, 10], True, 420, 10 ** 9, seg_count=cnt)
    assert cuts == [(0, 64), (3, 64)] and cnt == [1, 1, 1, 1, 0]
    # second transition: second selection of each (R_1 = 32); now the 50- and 40-token segments are cut to 32
    cuts = tbe.anneal_plan([R, E, T, E, R], [64, 50, 40, 64, 30], True, 248, 10 ** 9, seg_count=cnt)
    assert cuts == [(0, 32), (1, 32), (2, 32), (3, 32)] and cnt == [2, 2, 2, 2, 0]
    # three more transitions take every closed segment to the floor of 4; a sixth selects nothing any more
    live = [32, 32, 32, 32, 30]
    for want in (16, 8, 4):
        cuts = tbe.anneal_plan([R, E, T, E, R], live, True, sum(live), 10 ** 9, seg_count=cnt)
        assert cuts == [(i, want) for i in range(4)]
        live = [want] * 4 + [30]
    assert cnt == [5, 5, 5, 5, 0]
    assert tbe.anneal_plan([R, E, T, E, R], live, True, sum(live), 10 ** 9, seg_count=cnt) == [] and cnt == [5, 5, 5, 5, 0]
    # a segment that lost tokens in some other way keeps what it has when that is less than its level: |S*| = min(|S|, R_n)
    cnt = [1, 0]
    assert tbe.anneal_plan([E, R], [20, 7], True, 27, 10 ** 9, seg_count=cnt) == [] and cnt == [2, 0]
    # Case 2: over budget, no transition: least important type first (T, then E, then R), oldest first, one level per
    # selection, until the budget is met.  192 -> 64 -> 32, then the next transition segment; the 50-token E segment's
    # first selection removes nothing and is followed at once by its second
    cnt = [0, 0, 0, 0, 0]
    cuts = tbe.anneal_plan([E, T, T, R, E], [50, 192, 100, 128, 9], False, 479, 250, seg_count=cnt)
    # T segments: 1 (192 -> 64: 351 live, -> 32: 319, -> 16: 303, -> 8: 295, -> 4: 291), then 2 (100 -> 64: 255, -> 32: 223 <= 250)
    assert cuts == [(1, 64), (1, 32), (1, 16), (1, 8), (1, 4), (2, 64), (2, 32)] and cnt == [0, 5, 2, 0, 0]
    cnt = [0, 0, 0, 0, 0]
    cuts = tbe.anneal_plan([E, T, T, R, E], [50, 4, 4, 128, 9], False, 195, 150, seg_count=cnt)
    # the T segments cannot lose anything: five selections each that remove nothing; then E: 50 keeps 50 (n = 0), then 32: 177;
    # 16: 161; 8: 153; 4: 149
    assert cuts == [(0, 32), (0, 16), (0, 8), (0, 4)] and cnt == [5, 5, 5, 0, 0]
    # nothing can be selected any more: the plan stops even though the budget is not met
    assert tbe.anneal_plan([T, T, R], [4, 4, 500], False, 508, 100, seg_count=[5, 5, 0]) == []


def test_anneal_plan_where_count_and_size_rules_differ():
    T, E, R = 0, 1, 2
    # a 50-token segment, first selection: the paper's rule keeps all 50, the size-derived reading cuts to 32
    assert tbe.anneal_plan([E, R], [50, 5], True, 55, 10 ** 9, seg_count=[0, 0]) == []
    assert tbe.anneal_plan([E, R], [50, 5], True, 55, 10 ** 9, rule=tbe.BY_SIZE) == [(0, 32)]
    # a 192-token segment: the same first cut (64) under both; but a segment whose K-means run left 60 of 64 (a cluster
    # emptied) is cut to 32 under both on its second selection, while one left with exactly 64 ...
    assert tbe.anneal_plan([E, R], [192, 5], True, 197, 10 ** 9, seg_count=[0, 0]) == [(0, 64)]
    assert tbe.anneal_plan([E, R], [192, 5], True, 197, 10 ** 9, rule=tbe.BY_SIZE) == [(0, 64)]
    assert tbe.anneal_plan([E, R], [64, 5], True, 69, 10 ** 9, seg_count=[1, 0]) == [(0, 32)]
    assert tbe.anneal_plan([E, R], [64, 5], True, 69, 10 ** 9, rule=tbe.BY_SIZE) == [(0, 32)]
    # ... and one that grew after its first selection (cut to 64 while still open, 100 tokens now) goes to 32 by count, to 64 by size
    assert tbe.anneal_plan([E, R], [100, 5], True, 105, 10 ** 9, seg_count=[1, 0]) == [(0, 32)]
    assert tbe.anneal_plan([E, R], [100, 5], True, 105, 10 ** 9, rule=tbe.BY_SIZE) == [(0, 64)]
    # a segment with 30 tokens at count 1: by count it keeps min(30, 32) = 30, by size it is cut to 16
    cnt = [1, 0]
    assert tbe.anneal_plan([T, R], [30, 5], True, 35, 10 ** 9, seg_count=cnt) == [] and cnt == [2, 0]
    assert tbe.anneal_plan([T, R], [30, 5], True, 35, 10 ** 9, rule=tbe.BY_SIZE) == [(0, 16)]


def test_anneal_plan_by_size_option():
    T, E, R = 0, 1, 2
    size = dict(rule=tbe.BY_SIZE)
    # Case 1: a transition segment has just ended -> every earlier segment goes down one level; the open segment is left alone
    cuts = tbe.anneal_plan([R, E, T, R], [128, 100, 40, 10], True, 278, 10 ** 9, **size)
    assert cuts == [(0, 64), (1, 64), (2, 32)]
    # a second transition: next level each; a segment at the floor stays
    cuts = tbe.anneal_plan([R, E, T, R, T, E], [64, 64, 32, 4, 20, 7], True, 191, 10 ** 9, **size)
    assert cuts == [(0, 32), (1, 32), (2, 16), (4, 16)]
    # Case 2: least important type first, oldest first, one level at a time
    # 562 live, budget 400: T segment 128 -> 64 (498) -> 32 (466) -> 16 (450) -> 8 (442) -> 4 (438), then the oldest E segment 128 -> 64 (374)
    cuts = tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 400, **size)
    assert cuts == [(2, 64), (2, 32), (2, 16), (2, 8), (2, 4), (1, 64)]
    assert tbe.anneal_plan([T, T, R], [4, 4, 500], False, 508, 100, **size) == []


def test_anneal_plan_one_cut_per_segment_and_capacity():
    T, E, R = 0, 1, 2
    # over budget by a lot: with once=True the transition segment is cut once, then the plan moves on to the next candidates
    cnt = [0] * 5
    cuts = tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 300, once=True, seg_count=cnt)
    assert cuts == [(2, 64), (1, 64), (3, 64), (0, 64)] and cnt == [1, 1, 1, 1, 0]
    # capacity: stops after max_cuts cuts; a cut there is no room for leaves its segment's count alone
    cnt = [0] * 5
    assert tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 300, once=True, max_cuts=2, seg_count=cnt) == [(2, 64), (1, 64)]
    assert cnt == [0, 1, 1, 0, 0]
    # Case 1 and Case 2 in one call: the transition cut is not repeated by Case 2
    cnt = [0] * 4
    cuts = tbe.anneal_plan([T, R, T, E], [100, 100, 20, 9], True, 229, 60, once=True, seg_count=cnt)
    # Case 1: 100 -> 64, 100 -> 64, 20 keeps 20 (count 1).  157 live > 60.  Case 2: T first: segment 0 was cut in this call;
    # segment 2 (count 1 -> R_1 = 32: keeps 20, count 2 -> 16: cut); then E: none closed; R: segment 1 was cut in this call
    assert cuts == [(0, 64), (1, 64), (2, 16)] and cnt == [1, 1, 3, 0]
    # the size-derived option with once=True and a capacity
    assert tbe.anneal_plan([R, E, T, E, R], [128, 128, 128, 128, 50], False, 562, 300, once=True, max_cuts=2, rule=tbe.BY_SIZE) == [(2, 64), (1, 64)]


def test_plan_evictions_groups_live_tokens_by_segment_start():
    cfg = oc.OracleConfig(1, 8, 2, 64, (8, 2, 4), 1, 64, (64, 64, 64))
    c = oc.OracleCache(cfg)
    rng = np.random.default_rng(5)
    n = 300
    types = np.array([2] * 100 + [0] * 80 + [1] * 120, np.uint8)          # three segments: R, T, E (the last one open)
    k = rng.standard_normal((n, 2, 64)).astype(np.float16).astype(np.float32)
    h = np.asarray(c.append(0, k, k, np.zeros(n, np.int64), np.arange(n), types))
    c.evict_slots(0, [0] * 10, h[5:15])                                    # ten tokens of segment 0 are gone already
    cnt = [0, 0, 0]
    plan = tbe.plan_evictions(c, 0, 0, [0, 100, 180], [2, 0, 1], True, 10 ** 9, 8, seg_count=cnt)
    assert [(i, r) for i, r, _ in plan] == [(0, 64), (1, 64)] and cnt == [1, 1, 0]
    assert plan[0][2] == [int(x) for x in np.r_[h[:5], h[15:100]]]         # live tokens of the segment, ascending position
    assert plan[1][2] == [int(x) for x in h[100:180]]
    # no trigger, within budget: nothing
    assert tbe.plan_evictions(c, 0, 0, [0, 100, 180], [2, 0, 1], False, 290, 8) == []
    # over budget: the transition segment first (least important), then execution is open, so reasoning
    plan = tbe.plan_evictions(c, 0, 0, [0, 100, 180], [2, 0, 1], False, 200, 8)
    assert [(i, r) for i, r, _ in plan] == [(1, 64), (0, 64)]
