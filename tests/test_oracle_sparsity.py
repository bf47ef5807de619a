"""Pins for the oracle's attention-sparsity statistic (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import cache as oc
from oracle import sparsity as osp

LN100 = np.log(100.0)


def _cfg(bits=(8, 8, 8), D=64, H=2, G=4, seqs=1):
    return oc.OracleConfig(1, G * H, H, D, bits, seqs, 64, (64, 64, 64))


def _fill(cache, k, v, cls=None):
    n = k.shape[0]
    cls = np.zeros(n, np.uint8) if cls is None else cls
    return cache.append(0, k, v, np.zeros(n, np.int64), np.arange(n), cls)


def test_closed_forms_on_pooled_rows():
    # all scores equal: every weight equals the maximum, nothing is negligible
    assert osp.row_sparsity(np.full(37, 1.25)) == 0.0
    # one score far above the rest: all others are negligible
    r = np.zeros(50)
    r[7] = 40.0
    assert osp.row_sparsity(r) == 49 / 50
    # the boundary is ln(100) below the maximum in score units: just inside / just outside
    r = np.array([5.0, 5.0 - LN100 + 1e-9, 5.0 - LN100 - 1e-9, 5.0 - 10.0])
    assert osp.row_sparsity(r) == 2 / 4
    assert osp.row_sparsity(np.zeros(0)) == 0.0
    # shift invariance (softmax) and dependence on differences only
    rng = np.random.default_rng(0)
    r = rng.standard_normal(200) * 3
    assert osp.row_sparsity(r) == osp.row_sparsity(r + 123.0)


def test_row_sparsity_equals_library_softmax_count():
    """the definition through torch's own softmax: count entries below 1 % of the row maximum"""
    rng = np.random.default_rng(1)
    for n, spread in ((10, 1.0), (300, 2.0), (1000, 4.0)):
        r = rng.standard_normal(n) * spread
        w = torch.softmax(torch.from_numpy(r), dim=0).numpy()
        # keep clear of entries that sit on the boundary to within rounding
        assert np.abs(np.log(w / w.max()) + LN100).min() > 1e-9
        assert osp.row_sparsity(r) == np.count_nonzero(w < 0.01 * w.max()) / n


def test_pooling_is_the_groupwise_maximum_by_brute_force():
    rng = np.random.default_rng(2)
    Hkv, G, D, n = 2, 4, 16, 9
    q = rng.standard_normal((Hkv * G, D))
    k = rng.standard_normal((n, Hkv, D))
    pooled = osp.pooled_scores(q, k, 0.25)
    for h in range(Hkv):
        for j in range(n):
            best = max(0.25 * sum(q[h * G + g, d] * k[j, h, d] for d in range(D)) for g in range(G))
            assert abs(pooled[h, j] - best) < 1e-12


def test_single_query_head_per_group_is_plain_attention_sparsity():
    """G = 1: pooling does nothing, the statistic is the sparsity of the ordinary attention row,
    whose weights are exp(score - lse) with the lse of the attention oracle"""
    rng = np.random.default_rng(3)
    cfg = _cfg(G=1, H=2, D=64)
    c = oc.OracleCache(cfg)
    n = 120
    k = (rng.standard_normal((n, 2, 64)) * 2).astype(np.float16).astype(np.float32)
    v = rng.standard_normal((n, 2, 64)).astype(np.float16).astype(np.float32)
    _fill(c, k, v, rng.integers(0, 3, n).astype(np.uint8))
    q = rng.standard_normal((1, 2, 64))
    scale = 64 ** -0.5
    got = osp.decode_sparsity(c, 0, q, [0], [n], 0, scale)[0]
    _, lse = oa.decode_attention(c, 0, q, [0], [n], 0, scale)
    _, kd, _ = oa.gather_live(c, 0, 0)
    fr = []
    for h in range(2):
        w = np.exp(scale * (kd[:, h, :] @ q[0, h]) - lse[0, h])
        assert abs(w.sum() - 1) < 1e-12
        fr.append(np.count_nonzero(w < 0.01 * w.max()) / n)
    assert got == pytest.approx(np.mean(fr), abs=1e-15)


def test_constructed_cache_with_known_count():
    """keys that dequantise exactly (8-bit codes on the grid), a query along one channel: the
    pooled scores are known numbers and the count can be done by hand"""
    cfg = _cfg(bits=(8, 8, 8), G=4, H=1, D=64)
    c = oc.OracleCache(cfg)
    n = 16
    k = np.zeros((n, 1, 64), np.float32)
    k[:, 0, 0] = np.arange(n, dtype=np.float32)          # channel 0: 0, 1, ..., 15; group range 15 -> scale 15/255 exact? use channel 1 to pin the range
    k[:, 0, 1] = 255.0                                     # makes max - min = 255 in every token's first group: scale 1, codes = values
    v = np.zeros((n, 1, 64), np.float32)
    _fill(c, k, v)
    _, kd, _ = oa.gather_live(c, 0, 0)
    assert np.array_equal(kd[:, 0, 0], np.arange(n))       # stored exactly
    q = np.zeros((1, 4, 64))
    q[0, 0, 0], q[0, 1, 0], q[0, 2, 0], q[0, 3, 0] = 1.0, 0.5, -1.0, 0.25     # pooled over the group: max_g q_g * j = j for j >= 0
    got = osp.decode_sparsity(c, 0, q, [0], [n], 0, 1.0)[0]
    # scores 0..15, maximum 15, negligible below 15 - ln(100) = 10.39...: j = 0..10 -> 11 of 16
    assert got == 11 / 16
    # evicting the top three tokens moves the maximum to 12: negligible j <= 7 -> 8 of 13
    hs = [oc.make_handle(0, 0, 15), oc.make_handle(0, 0, 14), oc.make_handle(0, 0, 13)]
    c.evict_slots(0, [0, 0, 0], hs)
    assert osp.decode_sparsity(c, 0, q, [0], [n], 0, 1.0)[0] == 8 / 13
    # a window of 4 positions before the query at position 12: tokens 9..12 -> maximum 12, none negligible
    assert osp.decode_sparsity(c, 0, q, [0], [12], 4, 1.0)[0] == 0.0
    # nothing visible
    assert osp.decode_sparsity(c, 0, q, [0], [40], 4, 1.0)[0] == 0.0


def test_classify_orders_the_types_as_the_paper_observes():
    # densest -> execution (1), middle -> reasoning (2), sparsest -> transition (0)
    assert osp.classify(np.array([0.10, 0.50, 0.90]), (0.3, 0.7)).tolist() == [1, 2, 0]
    assert osp.classify(np.array([0.3, 0.7]), (0.3, 0.7)).tolist() == [2, 0]
