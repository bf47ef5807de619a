"""Pins for the oracle's decode attention (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import cache as oc
from oracle import quant

T, E, R = 0, 1, 2


def _cfg(bits=(8, 2, 4), D=64, H=2, G=4, seqs=2, layers=1):
    return oc.OracleConfig(layers, G * H, H, D, bits, seqs, 64, (64, 64, 64))


def _kv(n, H, D, seed, outliers=True):
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((n, H, D)).astype(np.float32)
    v = rng.standard_normal((n, H, D)).astype(np.float32)
    if outliers:
        for ch in (3, 17, D // 2 + 5, D - 2):
            k[..., ch] *= 8
            v[..., ch] *= 8
    f16 = lambda a: a.astype(np.float16).astype(np.float32)
    return f16(k), f16(v)


def _q(Hq, D, seed):
    return np.random.default_rng(1000 + seed).standard_normal((1, Hq, D)).astype(np.float16).astype(np.float64)


def _library_attention(q, k, v, scale, G):
    """softmax(q K^T * scale) V through torch's own softmax/matmul in binary64"""
    qt, kt, vt = (torch.from_numpy(np.ascontiguousarray(a)) for a in (q, k, v))
    out = []
    for h in range(q.shape[0]):
        a = torch.softmax((kt[:, h // G, :] @ qt[h]) * scale, dim=0)
        out.append(a @ vt[:, h // G, :])
    return torch.stack(out).numpy()


def _build(cfg, k, v, cls, order=None, seq=0):
    c = oc.OracleCache(cfg)
    n = len(cls)
    order = np.arange(n) if order is None else order
    h = c.append(0, k[order], v[order], np.full(n, seq), order, np.asarray(cls)[order])
    return c, h


def test_equals_library_softmax_on_the_dequantised_tensors():
    cfg = _cfg()
    n = 150
    k, v = _kv(n, 2, 64, 0)
    cls = np.random.default_rng(0).integers(0, 3, n)
    c, _ = _build(cfg, k, v, cls)
    q = _q(8, 64, 0)
    out, lse = oa.decode_attention(c, 0, q, [0], [n - 1], 0, 0.125)
    kh = np.zeros((n, 2, 64))
    vh = np.zeros((n, 2, 64))
    for i in range(n):                                   # dequantise token by token, independently
        b = cfg.bits_of_class[cls[i]]
        kc, ks, kz = quant.quantize_groups(k[i], b)
        vc, vs, vz = quant.quantize_groups(v[i], b)
        kh[i] = kz.astype(np.float64).repeat(32, -1) + kc * ks.astype(np.float64).repeat(32, -1)
        vh[i] = vz.astype(np.float64).repeat(32, -1) + vc * vs.astype(np.float64).repeat(32, -1)
    ref = _library_attention(q[0], kh, vh, 0.125, 4)
    assert np.abs(out[0] - ref).max() < 1e-12
    sc = 0.125 * (kh[:, 0, :] @ q[0, 1])
    assert abs(lse[0, 1] - torch.logsumexp(torch.from_numpy(sc), 0).item()) < 1e-12


def test_evicted_equals_masked_equals_absent():
    cfg = _cfg()
    n = 200
    k, v = _kv(n, 2, 64, 1)
    cls = np.random.default_rng(1).integers(0, 3, n)
    c, h = _build(cfg, k, v, cls)
    dead = np.random.default_rng(2).choice(n, 70, replace=False)
    c.evict_slots(0, [0] * 70, h[dead])
    keep = np.setdiff1d(np.arange(n), dead)
    c2 = oc.OracleCache(cfg)                               # a cache that never saw the dead tokens
    c2.append(0, k[keep], v[keep], np.zeros(len(keep), int), keep, cls[keep])
    q = _q(8, 64, 1)
    a, la = oa.decode_attention(c, 0, q, [0], [n], 0, 0.125)
    b, lb = oa.decode_attention(c2, 0, q, [0], [n], 0, 0.125)
    assert np.abs(a - b).max() <= 1e-12 and np.abs(la - lb).max() <= 1e-12


def test_invariant_to_physical_slot_permutation():
    """Theorem 'KV Permutation Invariance of Attention' and its GQA remark."""
    cfg = _cfg()
    n = 180
    k, v = _kv(n, 2, 64, 3)
    cls = np.random.default_rng(3).integers(0, 3, n)
    q = _q(8, 64, 3)
    ref, _ = oa.decode_attention(_build(cfg, k, v, cls)[0], 0, q, [0], [n], 0, 0.125)
    for seed in range(3):
        perm = np.random.default_rng(10 + seed).permutation(n)      # tokens arrive in another order
        c, _ = _build(cfg, k, v, cls, order=perm)
        got, _ = oa.decode_attention(c, 0, q, [0], [n], 0, 0.125)
        assert np.array_equal(got, ref)
    # scramble through eviction + reuse: junk tokens are placed, evicted, and real ones fill the holes
    c = oc.OracleCache(cfg)
    junk_k, junk_v = _kv(90, 2, 64, 99)
    jh = c.append(0, junk_k, junk_v, np.zeros(90, int), 1000 + np.arange(90), np.arange(90) % 3)
    c.append(0, k[:60], v[:60], np.zeros(60, int), np.arange(60), cls[:60])
    c.evict_slots(0, [0] * 90, jh)
    c.append(0, k[60:], v[60:], np.zeros(n - 60, int), np.arange(60, n), cls[60:])
    got, _ = oa.decode_attention(c, 0, q, [0], [n], 0, 0.125)
    assert np.array_equal(got, ref)


def test_closed_forms():
    cfg = _cfg()
    k, v = _kv(40, 2, 64, 4)
    q = _q(8, 64, 4)
    # one live token: output is that token's dequantised value row, exactly
    c, _ = _build(cfg, k[:1], v[:1], [R])
    out, lse = oa.decode_attention(c, 0, q, [0], [0], 0, 0.125)
    vh = quant.dequantize(*quant.quantize_groups(v[0], 4))
    for h in range(8):
        assert np.array_equal(out[0, h], vh[h // 4])
    # zero query: uniform weights -> the mean of the dequantised values; lse = log n
    c, _ = _build(cfg, k, v, [E] * 40)
    out, lse = oa.decode_attention(c, 0, np.zeros((1, 8, 64)), [0], [39], 0, 0.125)
    vh = quant.dequantize(*quant.quantize_groups(v, 2))
    assert np.abs(out[0, 5] - vh[:, 1, :].mean(0)).max() < 1e-13
    assert np.allclose(lse, np.log(40))
    # one dominant score: output tends to that token's value
    kd = k.copy()
    kd[7] = 0
    kd[7, :, 0] = 60000.0
    qd = np.zeros((1, 8, 64))
    qd[0, :, 0] = 50.0
    c, _ = _build(cfg, kd, v, [R] * 40)
    out, _ = oa.decode_attention(c, 0, qd, [0], [39], 0, 0.125)
    vh = quant.dequantize(*quant.quantize_groups(v, 4))
    assert np.abs(out[0, 0] - vh[7, 0]).max() < 1e-9
    # empty cache / everything evicted: zeros and -inf, no NaN
    c = oc.OracleCache(cfg)
    out, lse = oa.decode_attention(c, 0, q, [1], [0], 0, 0.125)
    assert not out.any() and np.all(np.isneginf(lse))


def test_gqa_head_mapping_and_per_head_softmax():
    """each query head gets its own softmax over its group's shared K/V (no max-pooling in
    the output path); heads 0..G-1 read kv head 0, the next G read kv head 1"""
    cfg = _cfg(bits=(8, 8, 8))
    k, v = _kv(30, 2, 64, 5, outliers=False)
    c, _ = _build(cfg, k, v, [T] * 30)
    q = _q(8, 64, 5)
    out, _ = oa.decode_attention(c, 0, q, [0], [29], 0, 0.125)
    kh = quant.dequantize(*quant.quantize_groups(k, 8))
    vh = quant.dequantize(*quant.quantize_groups(v, 8))
    for h in (0, 3, 4, 7):
        s = 0.125 * kh[:, h // 4, :] @ q[0, h]
        w = np.exp(s - s.max())
        w /= w.sum()
        assert np.abs(out[0, h] - w @ vh[:, h // 4, :]).max() < 1e-13
    assert np.abs(out[0, 0] - out[0, 4]).max() > 1e-3


def test_all_8bit_no_eviction_close_to_unquantised_attention():
    """With every class at 8 bits and nothing evicted the result is
    unquantised attention up to quantisation error; the bound below is first order and
    computed per case:  ds = max_j sum_i |q_i| s^K_ji / 2 * scale ;
    |o - o^| <= max|v - v^| + (e^{2 ds} - 1) * max|v^|."""
    cfg = _cfg(bits=(8, 8, 8), D=128)
    n = 300
    k, v = _kv(n, 2, 128, 6)
    cls = np.random.default_rng(6).integers(0, 3, n)
    c, _ = _build(cfg, k, v, cls)
    q = _q(8, 128, 6)
    scale = 128 ** -0.5
    out, _ = oa.decode_attention(c, 0, q, [0], [n], 0, scale)
    ref = _library_attention(q[0], k.astype(np.float64), v.astype(np.float64), scale, 4)
    kc, ks, kz = quant.quantize_groups(k, 8)
    vh = quant.dequantize(*quant.quantize_groups(v, 8))
    worst = 0.0
    for h in range(8):
        step = ks[:, h // 4, :].astype(np.float64).repeat(32, -1)
        ds = (np.abs(q[0, h])[None, :] * step / 2).sum(1).max() * scale
        bound = np.abs(v - vh).max() + np.expm1(2 * ds) * np.abs(vh).max()
        err = np.abs(out[0, h] - ref[h]).max()
        assert err <= bound
        worst = max(worst, err)
    assert worst < 0.1            # about one 8-bit step of an outlier group (range ~40 / 255 = 0.16)


def test_sliding_window_keeps_the_last_w_positions():
    cfg = _cfg()
    n = 100
    k, v = _kv(n, 2, 64, 7)
    cls = np.random.default_rng(7).integers(0, 3, n)
    c, h = _build(cfg, k, v, cls)
    q = _q(8, 64, 7)
    W = 32
    out, _ = oa.decode_attention(c, 0, q, [0], [n - 1], W, 0.125)
    keep = np.arange(n - W, n)
    c2 = oc.OracleCache(cfg)
    c2.append(0, k[keep], v[keep], np.zeros(W, int), keep, cls[keep])
    ref, _ = oa.decode_attention(c2, 0, q, [0], [n - 1], 0, 0.125)
    assert np.abs(out - ref).max() < 1e-13


def test_split_merge_identity():
    """cutting the context into chunks and merging per-chunk (m, l, acc) by log-sum-exp gives the
    same result for any chunking -- the identity the split-K path relies on"""
    cfg = _cfg()
    n = 130
    k, v = _kv(n, 2, 64, 8)
    c, _ = _build(cfg, k, v, [R] * n)
    q = _q(8, 64, 8)
    ref, lse_ref = oa.decode_attention(c, 0, q, [0], [n], 0, 0.125)
    _, kh, vh = oa.gather_live(c, 0, 0)
    for chunk in (1, 7, 16, 64, 130):
        parts = [oa.attend_dense(q[0], kh[i:i + chunk], vh[i:i + chunk], 0.125) for i in range(0, n, chunk)]
        lses = np.stack([p[1] for p in parts])
        M = lses.max(0)
        w = np.exp(lses - M)
        o = sum(w[i][:, None] * parts[i][0] for i in range(len(parts))) / w.sum(0)[:, None]
        assert np.abs(o - ref[0]).max() < 1e-12
        assert np.abs(M + np.log(w.sum(0)) - lse_ref[0]).max() < 1e-12
