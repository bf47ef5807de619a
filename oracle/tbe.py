"""Thought-adaptive eviction over the oracle cache: which tokens of a thought segment survive
(test infrastructure; see oracle/__init__.py).

Sec. 4.3 of the paper ("Think Before you Evict"), problem statement "Thought-Adaptive Eviction":
a segment that is selected for eviction the n-th time keeps min(|segment|, R_n) tokens,
R = {64, 32, 16, 8, 4}; the survivors are chosen by K-means over the segment's post-RoPE keys
with that K, one representative key of every cluster staying in the cache together with its
value (appendix "TBE Eviction Policy").  Case 1 anneals every preceding segment when a
transition segment ends; Case 2, when the cache is over its budget, anneals the oldest segment
of the least important type until it fits.

The paper fixes neither the K-means variant, its initialisation, its stopping rule nor any
tie-break.  This reading (the kernels implement the same one):

  points      x_i = the token's stored keys, dequantised (zp + code * scale), all kv-heads
              concatenated: eviction is per token, so one clustering serves all heads; tokens
              in ascending position
  K >= N      everything survives
  init        centroid j = point floor(j * N / K)  (evenly spaced over the segment)
  Lloyd       assign every point to its nearest centroid (squared Euclidean distance; ties ->
              lowest cluster); stop when no assignment changed or after max_iters assignments;
              otherwise move every centroid to the mean of its points (a cluster that lost all
              its points keeps its centroid) and repeat
  survivors   of every non-empty cluster the point nearest its centroid (ties -> lowest index; a
              cluster of two points, both equally near their mean whatever the rounding says,
              keeps the earlier one); so at most K tokens survive, exactly K when no cluster is
              empty

Everything in binary64.  The decisions are comparisons of floating-point numbers; `margin`
reports how close the closest one was, so that a test can tell a genuine disagreement with a
binary32 implementation from a coin toss.
"""
import numpy as np

from . import quant
from .cache import split_handle

RETENTION = (64, 32, 16, 8, 4)
IMPORTANCE = (0, 1, 2)      # least important first: transition, execution, reasoning (Sec. 4.1 / 4.2 ordering)


def _sqdist(x, c):
    """[N, K] squared distances, written out (no expansion into norms and dot products)"""
    d = x[:, None, :] - c[None, :, :]
    return np.einsum("nkd,nkd->nk", d, d)


def kmeans_select(x, keep, max_iters=8):
    """x [N, dim] binary64, points in segment order.  Returns (survivors: sorted indices,
    margin: smallest gap between the best and the second-best candidate over all decisions,
    relative to the mean squared norm of the points, objective after every assignment)."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    k = min(n, int(keep))
    if k >= n:
        return np.arange(n), np.inf, []
    cent = x[(np.arange(k) * n) // k].copy()
    scale = max(float(np.mean(np.einsum("nd,nd->n", x, x))), 1e-300)
    margin = np.inf
    prev = None
    objective = []
    for _ in range(max_iters):
        d = _sqdist(x, cent)
        assign = np.argmin(d, axis=1)                      # first minimum: ties -> lowest cluster
        if k > 1:
            two = np.partition(d, 1, axis=1)[:, :2]
            margin = min(margin, float((two[:, 1] - two[:, 0]).min()) / scale)
        objective.append(float(d[np.arange(n), assign].sum()))
        if prev is not None and np.array_equal(assign, prev):
            break
        for j in range(k):
            members = np.flatnonzero(assign == j)
            if members.size:
                cent[j] = x[members].mean(axis=0)
        prev = assign
    d = _sqdist(x, cent)
    survivors = []
    for j in range(k):
        members = np.flatnonzero(prev == j)
        if members.size == 0:
            continue
        if members.size <= 2:
            survivors.append(int(members[0]))              # two points are equally near their mean: the earlier one
            continue
        dj = d[members, j]
        survivors.append(int(members[np.argmin(dj)]))      # first minimum: ties -> lowest index
        two = np.partition(dj, 1)[:2]
        margin = min(margin, float(two[1] - two[0]) / scale)
    return np.array(sorted(survivors), dtype=np.int64), margin, objective


def segment_keys(cache, layer, seq, handles):
    """dequantised keys [N, Hkv * D] (binary64) of the listed slots of one sequence"""
    H, D = cache.cfg.n_kv_heads, cache.cfg.head_dim
    out = np.zeros((len(handles), H * D))
    for i, h in enumerate(handles):
        c, pi, slot = split_handle(h)
        pid = int(cache.table[seq, layer, c, pi])
        out[i] = cache.dequant(c, 0, np.array([pid]), np.array([slot])).reshape(-1)
    return out


def select_evictions(cache, layer, tok_seq, tok_handle, seg_offset, seg_keep, max_iters=8):
    """The call the kernels implement: segments given as runs [seg_offset[s], seg_offset[s+1]) of
    (sequence, handle) lists, tokens of a segment in ascending position.  Returns (ev_handle
    [n_tok]: the handle of every token to evict, -1 for a survivor; margins [n_seg]: the
    smallest margin met inside each segment)."""
    tok_handle = np.asarray(tok_handle, dtype=np.int64)
    ev = tok_handle.copy()
    margins = np.full(len(seg_keep), np.inf)
    for s in range(len(seg_keep)):
        lo, hi = int(seg_offset[s]), int(seg_offset[s + 1])
        if hi <= lo:
            continue
        x = segment_keys(cache, layer, int(tok_seq[lo]), tok_handle[lo:hi])
        keep, margins[s], _ = kmeans_select(x, int(seg_keep[s]), max_iters)
        ev[lo + keep] = -1
    return ev.astype(np.int32), margins


BY_COUNT, BY_SIZE = "count", "size"


def anneal_plan(seg_type, seg_live, transition_ended, n_live, budget, retention=RETENTION, importance=IMPORTANCE,
                once=False, max_cuts=None, seg_count=None, rule=BY_COUNT):
    """Which segments of one (sequence, layer) are cut, and to how many tokens (Sec. 4.3).

    seg_type[i], seg_live[i]: thought type and live tokens of segment i, oldest first; the last
    segment is the one being generated and is never touched.

    rule BY_COUNT (the paper's statement of the problem): seg_count[i] = n, how often segment i has
    been selected so far (updated in place; zeros when not given).  A selection keeps
    min(live, R_n) tokens and makes the count n + 1; a segment can be selected while n is below
    the number of retention levels.  A selection that removes nothing (the segment is no larger
    than R_n) is not a cut: it only advances the count.
    rule BY_SIZE (a reading for callers that keep no counts): the level follows from the
    segment's size, which is cut to the largest retention value below it; seg_count is not used.

    Case 1 (transition_ended): every preceding segment is selected once.  Case 2: while more than
    `budget` tokens are live, the oldest segment of the least important type that can still be
    selected is.  Returns [(segment, keep)] in the order the cuts are made; a segment may appear
    twice.  once=True: a segment is cut at most once per call (one K-means per segment and call;
    what is still over budget is dealt with on the next call); max_cuts: at most that many cuts
    (a cut there is no room for is not made, and its selection does not count)."""
    live = [int(v) for v in seg_live]
    total = int(n_live)
    cuts = []
    levels = len(retention)
    if rule == BY_COUNT and seg_count is None:
        seg_count = [0] * len(live)

    def selectable(i):
        if rule == BY_COUNT:
            return seg_count[i] < levels
        return any(r < live[i] for r in retention)

    def target(i):
        """tokens segment i keeps if it is selected now"""
        if rule == BY_COUNT:
            return min(live[i], retention[seg_count[i]])
        return next(r for r in retention if r < live[i])

    last = len(live) - 1
    done = set()
    room = (lambda: True) if max_cuts is None else (lambda: len(cuts) < max_cuts)

    def select(i):
        """True if the selection was made (a cut, or a selection that removes nothing)"""
        nonlocal total
        r = target(i)
        if r < live[i]:
            if not room():
                return False
            cuts.append((i, r))
            done.add(i)
            total -= live[i] - r
            live[i] = r
        if rule == BY_COUNT:
            seg_count[i] += 1
        return True

    if transition_ended:
        for i in range(last):
            if selectable(i):
                select(i)
    while total > budget and room():
        pick = None
        for t in importance:
            for i in range(last):
                if seg_type[i] == t and selectable(i) and not (once and i in done):
                    pick = i
                    break
            if pick is not None:
                break
        if pick is None:
            break
        if not select(pick):
            break
    return cuts


def plan_evictions(cache, layer, seq, seg_start, seg_type, transition_ended, budget, max_cuts, retention=RETENTION,
                   seg_count=None, rule=BY_COUNT):
    """The plan over the cache as it stands: every live token of the sequence belongs to the
    segment whose start is the largest one not above its position (the block table's start-index
    column, Sec. 5.2); segments are counted, anneal_plan (one cut per segment and call) names the
    cuts, and each cut comes with the handles of its live tokens in ascending position -- the
    input of the survivor choice.  seg_count (rule BY_COUNT): the segments' selection counts, updated
    in place.  Returns [(segment, keep, handles)]."""
    from .cache import make_handle, PAGE
    seg_start = np.asarray(seg_start, dtype=np.int64)
    n_seg = len(seg_start)
    members = [[] for _ in range(n_seg)]
    for c in range(3):
        for pi in range(int(cache.n_pages[seq, layer, c])):
            pid = int(cache.table[seq, layer, c, pi])
            m = int(cache.valid[c][pid])
            for slot in range(PAGE):
                if m >> slot & 1:
                    pos = int(cache.slot_pos[c][pid, slot])
                    sg = int(np.searchsorted(seg_start, pos, side="right")) - 1
                    if sg >= 0:
                        members[sg].append((pos, make_handle(c, pi, slot)))
    live = [len(m) for m in members]
    cuts = anneal_plan(list(seg_type), live, bool(transition_ended), int(cache.n_live[seq, layer]), budget,
                       retention=retention, once=True, max_cuts=max_cuts, seg_count=seg_count, rule=rule)
    return [(i, r, [h for _, h in sorted(members[i])]) for i, r in cuts]
