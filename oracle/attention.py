"""Decode attention over the oracle cache (test infrastructure; see oracle/__init__.py).

The method reaches exactly dense softmax attention over the retained, dequantised set, so
the oracle is that definition written out (appendix "Decode":  A = softmax(q K^T / sqrt(d)),
O = A V; "Grouped-Query Attention": the G query heads of a group share (K_h, V_h) and each
query head gets its own softmax -- the max-pool aggregation printed there is used by the
paper for its sparsity statistic only).  Everything is binary64:

    live set   = slots whose live bit is set [and 0 <= q_pos - slot_pos < W on window layers]
    k^_j, v^_j = the stored codes decoded with the STORED scales (zp + code * scale from the binary16 scale /
                 zero-point of the integer formats; code value times E4M3 or tensor scale for the paper's formats)
    o_h        = sum_j softmax_j(scale * q_h . k^_j) v^_j ,  lse_h = log sum_j exp(scale * q_h . k^_j)

Tokens are visited in ascending logical position (ties: table order), which makes the result
independent of where a token physically sits (Theorem "KV Permutation Invariance of
Attention").  An empty live set gives o = 0 and lse = -inf.
"""
import numpy as np


def gather_live(cache, s, layer, q_pos=None, window=0):
    """Returns (pos [n], k^ [n, Hkv, D], v^ [n, Hkv, D]) in binary64, sorted by position."""
    toks = cache.live_tokens(s, layer)
    if window > 0:
        toks = [t for t in toks if 0 <= q_pos - t[0] < window]
    H, D = cache.cfg.n_kv_heads, cache.cfg.head_dim
    n = len(toks)
    pos = np.array([t[0] for t in toks], dtype=np.int64)
    k = np.zeros((n, H, D))
    v = np.zeros((n, H, D))
    cls = np.array([t[1] for t in toks], dtype=np.int64)
    pid = np.array([t[2] for t in toks], dtype=np.int64)
    slot = np.array([t[3] for t in toks], dtype=np.int64)
    for c in range(3):
        sel = np.flatnonzero(cls == c)
        if sel.size == 0:
            continue
        p, sl = pid[sel], slot[sel]
        k[sel] = cache.dequant(c, 0, p, sl)
        v[sel] = cache.dequant(c, 1, p, sl)
    order = np.argsort(pos, kind="stable")
    return pos[order], k[order], v[order]


def attend_dense(q, k, v, scale):
    """q [Hq, D], k/v [n, Hkv, D] binary64 -> (o [Hq, D], lse [Hq])."""
    Hq, D = q.shape
    n, Hkv, _ = k.shape
    G = Hq // Hkv
    o = np.zeros((Hq, D))
    lse = np.full(Hq, -np.inf)
    if n == 0:
        return o, lse
    for h in range(Hq):
        kh, vh = k[:, h // G, :], v[:, h // G, :]
        sc = scale * (kh @ q[h])
        m = sc.max()
        p = np.exp(sc - m)
        l = p.sum()
        o[h] = (p / l) @ vh
        lse[h] = m + np.log(l)
    return o, lse


def decode_attention(cache, layer, q, seq_ids, q_pos, window, scale):
    """q: [B, Hq, D]; returns (out [B, Hq, D], lse [B, Hq]) in binary64."""
    q = np.asarray(q, dtype=np.float64)
    B, Hq, D = q.shape
    out = np.zeros((B, Hq, D))
    lse = np.full((B, Hq), -np.inf)
    for b in range(B):
        _, k, v = gather_live(cache, int(seq_ids[b]), layer, int(q_pos[b]), window)
        out[b], lse[b] = attend_dense(q[b], k, v, scale)
    return out, lse
