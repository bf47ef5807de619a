"""Attention-sparsity statistic of a decode step over the oracle cache (test infrastructure;
see oracle/__init__.py).

The paper identifies the thought type of a decode step from how sparse the step's normalised
attention scores are (Sec. 4.1; footnote there: the scores are softmax-normalised and an
entry counts as negligible when it lies below 1 % of the maximum of its row; appendix
"Grouped-Query Attention": for a group of G query heads sharing (K_h, V_h) the scaled scores
of the G heads are max-pooled element-wise over the group, the pooled row is renormalised by a
softmax along the keys, and the statistic is averaged over the groups).  Written out, for one
query of sequence s on one layer, in binary64:

    live set     = as for attention (live bit set [and inside the window on window layers])
    a_{h,g}[j]   = scale * q_{h,g} . k^_j                        g = 0..G-1, j in the live set
    pooled_h[j]  = max_g a_{h,g}[j]
    w_h          = softmax_j(pooled_h)
    sparsity_h   = #{ j : w_h[j] < 0.01 * max_j w_h[j] } / #live          (0 for an empty set)
    sparsity     = mean_h sparsity_h

The thresholds that turn the statistic into a thought type come from calibration data (Sec.
4.1 "Offline Calibration") and are inputs here: classify() compares against them.
"""
import numpy as np

from . import attention

NEGLIGIBLE = 0.01   # fraction of the row maximum below which an entry counts as zero


def pooled_scores(q, k, scale):
    """q [Hq, D], k [n, Hkv, D] binary64 -> pooled [Hkv, n]: the group-wise max of the scaled scores."""
    Hq, D = q.shape
    n, Hkv, _ = k.shape
    G = Hq // Hkv
    pooled = np.full((Hkv, n), -np.inf)
    for h in range(Hkv):
        for g in range(G):
            pooled[h] = np.maximum(pooled[h], scale * (k[:, h, :] @ q[h * G + g]))
    return pooled


def row_sparsity(pooled_row):
    """fraction of the softmax of one pooled row that lies below 1 % of the row's maximum"""
    n = pooled_row.shape[0]
    if n == 0:
        return 0.0
    e = np.exp(pooled_row - pooled_row.max())
    w = e / e.sum()
    return float(np.count_nonzero(w < NEGLIGIBLE * w.max())) / n


def decode_sparsity(cache, layer, q, seq_ids, q_pos, window, scale):
    """q: [B, Hq, D]; returns sparsity [B] in binary64."""
    q = np.asarray(q, dtype=np.float64)
    B = q.shape[0]
    out = np.zeros(B)
    for b in range(B):
        _, k, _ = attention.gather_live(cache, int(seq_ids[b]), layer, int(q_pos[b]), window)
        pooled = pooled_scores(q[b], k, scale)
        out[b] = float(np.mean([row_sparsity(pooled[h]) for h in range(pooled.shape[0])]))
    return out


def classify(sparsity, thresholds):
    """Thought type from the statistic and the calibrated thresholds theta_1 < theta_2 (Sec. 4.1
    Observation 1b: transition thoughts are the sparsest, execution thoughts the densest):
    0 = transition, 1 = execution, 2 = reasoning, the numbering of the paper's pseudocode."""
    lo, hi = thresholds
    s = np.asarray(sparsity)
    return np.where(s >= hi, 0, np.where(s < lo, 1, 2)).astype(np.int64)
