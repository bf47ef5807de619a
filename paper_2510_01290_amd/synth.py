"""Seeded synthetic workloads (inputs only -- no quantisation, paging or attention arithmetic).

Serves both the HIP path and the CPU oracle: it emits token streams (K/V rows, sequence id,
logical position, thought class), eviction lists (by logical position) and queries, as a
"script" of operations that any cache backend can replay.  The stand-in recipe follows the
shapes the paper works with (thought segments of about a hundred to a few hundred tokens,
three thought types, Sec. 4.1 / 5; cache budgets of 1-2K tokens and 32K-token generations,
Sec. 6), not its datasets.

Random values come from a counter-based generator built from integer operations and one
table lookup, so the same values can be produced on the CPU or on the GPU, for any
(sequence, layer) on its own:  u = hash32(counter, key) >> 16 ;  x = Phi^-1((u + 1/2) / 65536).
"""
from dataclasses import dataclass, field
import numpy as np
import torch

T, E, R = 0, 1, 2          # thought classes, numbered as in the paper's pseudocode
PAGE = 16
_M32 = 0xFFFFFFFF


def outlier_channels(D):
    return (3, 17, D // 2 + 5, D - 2)


_TABLE = {}


def _normal_table(device):
    key = str(device)
    if key not in _TABLE:
        from scipy.special import ndtri
        t = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0).astype(np.float32)
        _TABLE[key] = torch.from_numpy(t).to(device)
    return _TABLE[key]


def _mix(key_parts):
    """host-side 31-bit key from a tuple of small integers"""
    h = 0x9E3779B1
    for p in key_parts:
        h = ((h ^ (int(p) & _M32)) * 0x85EBCA6B) & _M32
        h ^= h >> 13
        h = (h * 0xC2B2AE35) & _M32
        h ^= h >> 16
    return h & 0x7FFFFFFF


def _hash32(idx, key):
    """idx: int64 tensor of counters (< 2^31); every product stays below 2^63."""
    h = (idx ^ key) & _M32
    h = ((h >> 16) ^ h) * 0x45D9F3B & _M32
    h = ((h >> 16) ^ h) * 0x45D9F3B & _M32
    h = (h >> 16) ^ h
    return h


def normals(key_parts, start, count, device):
    """float32 tensor [count]: standard-normal quantile-table draws for counters start.."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    u = _hash32(idx, _mix(key_parts)) >> 16
    return _normal_table(device)[u]


def torch_dtype(name):
    return {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[name]


@dataclass
class Geometry:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str = "bf16"                    # dtype of K/V rows and queries
    bits_of_class: tuple = (8, 2, 4)       # (T, E, R) -- BASELINE configs: T=8, R=4, E=2
    fmt: str = "int"                       # "int": integer codes, group 32 (BASELINE); "fp": the paper's E4M3 / NVFP4 / ternary
    fp8_scale: tuple = (0.05, 0.05)        # fmt "fp": per-tensor scales of keys and values of the 8-bit type


def kv_rows(seed, layer, seq, kind, t0, t1, geom, device):
    """K (kind=0) or V (kind=1) rows of logical tokens t0..t1-1 of one sequence:
    N(0,1) draws, four fixed outlier channels per head scaled by 8, rounded to geom.dtype."""
    H, D = geom.n_kv_heads, geom.head_dim
    x = normals((seed, 11, layer, seq, kind), t0 * H * D, (t1 - t0) * H * D, device).view(t1 - t0, H, D)
    scale = torch.ones(D, dtype=torch.float32, device=device)
    scale[list(outlier_channels(D))] = 8.0
    return (x * scale).to(torch_dtype(geom.dtype))


def query_rows(seed, layer, seq, step, geom, device):
    Hq, D = geom.n_q_heads, geom.head_dim
    x = normals((seed, 13, layer, seq, step), 0, Hq * D, device).view(Hq, D)
    return x.to(torch_dtype(geom.dtype))


def thought_classes(rng, n_tokens, p_ter=(0.2, 0.4, 0.4)):
    """Per-token class and segment id: segment lengths U{64..192}, labels T/E/R with
    probabilities p_ter (paper order T=0, E=1, R=2), drawn until n_tokens are covered."""
    cls = np.empty(n_tokens, dtype=np.uint8)
    seg = np.empty(n_tokens, dtype=np.int32)
    t, i = 0, 0
    while t < n_tokens:
        ln = int(rng.integers(64, 193))
        c = int(rng.choice(3, p=p_ter))
        cls[t:t + ln] = c
        seg[t:t + ln] = i
        t += ln
        i += 1
    return cls, seg


# ----------------------------------------------------------------------------- scripts
@dataclass
class Append:
    layer: int
    seqs: np.ndarray        # [m] sequence ids, ascending
    t0: np.ndarray          # [m] first logical position appended for that sequence
    cnt: np.ndarray         # [m] number of consecutive positions


@dataclass
class Evict:
    layer: int
    seqs: np.ndarray        # [n] sequence id of each evicted token
    pos: np.ndarray         # [n] logical position of each evicted token


@dataclass
class Workload:
    name: str
    geom: Geometry
    seed: int
    n_seqs: int
    classes: list           # per sequence: uint8 [max logical tokens] thought class of each position
    ops: list               # Append / Evict in execution order
    window_of_layer: tuple = ()     # 0 = full attention
    q_pos: np.ndarray = None        # [n_seqs] logical position of the decode query (last appended)

    def max_tokens(self):
        return max(len(c) for c in self.classes)


class ScriptRunner:
    """Replays a workload's ops on a backend with
         .device
         .append(layer, k, v, tok_seq, tok_pos, tok_class) -> int32 handles [n] (numpy)
         .evict(layer, ev_seq, ev_handle)
    keeping, per backend, the handle each logical position received."""

    def __init__(self, wl, backend, layers=None, seqs=None):
        self.wl, self.be = wl, backend
        self.with_data = getattr(backend, "needs_data", True)     # a backend that keeps tables only is not sent K/V rows
        self.layers = set(range(wl.geom.n_layers)) if layers is None else set(layers)
        self.seqs = None if seqs is None else set(int(s) for s in seqs)
        self.handle = {(l, s): np.full(len(wl.classes[s]), -1, dtype=np.int32)
                       for l in self.layers for s in range(wl.n_seqs)
                       if self.seqs is None or s in self.seqs}

    def tokens_of(self, op):
        """(tok_seq, tok_pos, tok_class, k, v) of an Append, restricted to the selected sequences"""
        wl, dev = self.wl, self.be.device
        ts, tp, tc, ks, vs = [], [], [], [], []
        for s, t0, n in zip(op.seqs.tolist(), op.t0.tolist(), op.cnt.tolist()):
            if n == 0 or (self.seqs is not None and s not in self.seqs):
                continue
            ts.append(np.full(n, s, dtype=np.int32))
            tp.append(np.arange(t0, t0 + n, dtype=np.int32))
            tc.append(wl.classes[s][t0:t0 + n])
            if self.with_data:
                ks.append(kv_rows(wl.seed, op.layer, s, 0, t0, t0 + n, wl.geom, dev))
                vs.append(kv_rows(wl.seed, op.layer, s, 1, t0, t0 + n, wl.geom, dev))
        if not ts:
            return None
        return (np.concatenate(ts), np.concatenate(tp), np.concatenate(tc).astype(np.uint8),
                torch.cat(ks) if self.with_data else None, torch.cat(vs) if self.with_data else None)

    def run(self, ops=None):
        for op in (self.wl.ops if ops is None else ops):
            if op.layer not in self.layers:
                continue
            if isinstance(op, Append):
                tk = self.tokens_of(op)
                if tk is None:
                    continue
                ts, tp, tc, k, v = tk
                h = np.asarray(self.be.append(op.layer, k, v, ts, tp, tc), dtype=np.int32)
                for s in np.unique(ts).tolist():
                    m = ts == s
                    self.handle[(op.layer, s)][tp[m]] = h[m]
            else:
                if self.seqs is not None:
                    m = np.isin(op.seqs, list(self.seqs))
                    seqs, pos = op.seqs[m], op.pos[m]
                else:
                    seqs, pos = op.seqs, op.pos
                if len(seqs) == 0:
                    continue
                hs = np.empty(len(seqs), dtype=np.int32)
                for s in np.unique(seqs).tolist():
                    m = seqs == s
                    hs[m] = self.handle[(op.layer, s)][pos[m]]
                self.be.evict(op.layer, seqs.astype(np.int32), hs)
        return self

    def queries(self, layer, step=0):
        wl = self.wl
        sel = sorted(self.seqs) if self.seqs is not None else range(wl.n_seqs)
        return torch.stack([query_rows(wl.seed, layer, s, step, wl.geom, self.be.device) for s in sel])


# ------------------------------------------------------------------ workload builders
def _evict_fraction(rng, live_pos, cls, frac_by_class):
    """positions to evict: for each class, a uniform sample without replacement of
    round(frac * n_live_of_class) of its live positions"""
    out = []
    for c, f in frac_by_class.items():
        cand = live_pos[cls[live_pos] == c]
        n = int(round(f * len(cand)))
        if n:
            out.append(rng.choice(cand, size=n, replace=False))
    return np.sort(np.concatenate(out)) if out else np.zeros(0, dtype=np.int64)


def bulk_evict_refill(name, geom, seed, n_seqs, ctx_tokens, evict_frac, refill=None,
                      refill_chunk=1, window_of_layer=None):
    """Configs 1, 2, 2* and 4: append ctx_tokens[s] tokens in bulk, evict a class-wise fraction
    of the live tokens (independently per layer), then append `refill` more tokens per sequence
    (None = as many as were evicted in layer 0), refill_chunk tokens per sequence per call."""
    rng = np.random.default_rng(seed)
    ctx = np.broadcast_to(np.asarray(ctx_tokens), (n_seqs,)).astype(np.int64)
    L = geom.n_layers
    ev = {}
    n_ref = np.zeros(n_seqs, dtype=np.int64)
    pre_classes = []
    for s in range(n_seqs):
        cls, _ = thought_classes(rng, int(ctx[s]))
        pre_classes.append(cls)
    for l in range(L):
        for s in range(n_seqs):
            ev[(l, s)] = _evict_fraction(rng, np.arange(ctx[s]), pre_classes[s], evict_frac)
    for s in range(n_seqs):
        n_ref[s] = len(ev[(0, s)]) if refill is None else refill
    classes = []
    for s in range(n_seqs):
        more, _ = thought_classes(rng, int(n_ref[s])) if n_ref[s] else (np.zeros(0, np.uint8), None)
        classes.append(np.concatenate([pre_classes[s], more[:n_ref[s]]]))
    ops = []
    seqs = np.arange(n_seqs, dtype=np.int32)
    for l in range(L):
        ops.append(Append(l, seqs, np.zeros(n_seqs, np.int64), ctx.copy()))
        es = np.concatenate([np.full(len(ev[(l, s)]), s, dtype=np.int32) for s in range(n_seqs)])
        ep = np.concatenate([ev[(l, s)] for s in range(n_seqs)])
        if len(es):
            ops.append(Evict(l, es, ep))
        done = np.zeros(n_seqs, dtype=np.int64)
        while (done < n_ref).any():
            cnt = np.minimum(refill_chunk, n_ref - done)
            ops.append(Append(l, seqs, ctx + done, cnt))
            done = done + cnt
    wol = tuple([0] * L) if window_of_layer is None else tuple(window_of_layer)
    return Workload(name, geom, seed, n_seqs, classes, ops, wol, (ctx + n_ref - 1).astype(np.int32))


def budgeted_decode(name, geom, seed, n_seqs, n_steps, budget, steps_per_call=16,
                    retention=(64, 32, 16, 8, 4), evict_order=(E, R, T)):
    """Config 3: n_steps decode appends per sequence under a live-token budget.  Whenever a
    sequence holds more than `budget` live tokens, the oldest closed segment of the least
    important class that can still be selected is: its n-th selection keeps min(size,
    retention[n]) tokens, chosen by a seeded uniform pick (the paper's budget case of
    thought-adaptive eviction, Sec. 4.3, with the K-means pick replaced by a random one); the
    segment being generated is never touched.  All layers share the token classes; eviction
    choices are drawn per layer."""
    rng = np.random.default_rng(seed)
    L = geom.n_layers
    classes, segs = [], []
    for s in range(n_seqs):
        c, g = thought_classes(rng, n_steps)
        classes.append(c)
        segs.append(g)
    ops = []
    seqs = np.arange(n_seqs, dtype=np.int32)
    for l in range(L):
        # per sequence: segment id -> live positions
        live = [dict() for _ in range(n_seqs)]
        selected = [dict() for _ in range(n_seqs)]     # segment id -> times selected so far
        n_live = np.zeros(n_seqs, dtype=np.int64)
        t = 0
        while t < n_steps:
            n = min(steps_per_call, n_steps - t)
            ops.append(Append(l, seqs, np.full(n_seqs, t, np.int64), np.full(n_seqs, n, np.int64)))
            es, ep = [], []
            for s in range(n_seqs):
                sg = segs[s][t:t + n]
                for g in np.unique(sg).tolist():
                    live[s].setdefault(g, []).extend((t + np.flatnonzero(sg == g)).tolist())
                n_live[s] += n
                open_seg = int(segs[s][t + n - 1])
                while n_live[s] > budget:
                    pick = None
                    for c in evict_order:
                        for g in sorted(live[s]):
                            if g == open_seg or classes[s][live[s][g][0]] != c:
                                continue
                            # selections that remove nothing only advance the segment's count
                            while selected[s].get(g, 0) < len(retention) and retention[selected[s].get(g, 0)] >= len(live[s][g]):
                                selected[s][g] = selected[s].get(g, 0) + 1
                            if selected[s].get(g, 0) < len(retention):
                                pick = (g, selected[s].get(g, 0))
                                break
                        if pick:
                            break
                    if pick is None:
                        break
                    g, lv = pick
                    selected[s][g] = lv + 1
                    keep = retention[lv]
                    cur = np.array(live[s][g])
                    drop = rng.choice(cur, size=len(cur) - keep, replace=False)
                    live[s][g] = sorted(set(cur.tolist()) - set(drop.tolist()))
                    n_live[s] -= len(drop)
                    es.append(np.full(len(drop), s, dtype=np.int32))
                    ep.append(np.sort(drop))
            if es:
                ops.append(Evict(l, np.concatenate(es), np.concatenate(ep)))
            t += n
    return Workload(name, geom, seed, n_seqs, classes, ops, tuple([0] * L),
                    np.full(n_seqs, n_steps - 1, dtype=np.int32))


# ------------------------------------------------------------------ the named configs
def config_tiny(seed=0, bits_of_class=(8, 2, 4)):
    g = Geometry(1, 8, 2, 64, "f16", bits_of_class)
    return bulk_evict_refill("cfg1-tiny", g, seed, 1, 1024, {E: 0.25}, refill=256)


def config_llama8b_layer(seed=1, n_seqs=16, ctx=8192, refill_chunk=1, name="cfg2-r1-llama-8b-layer"):
    g = Geometry(1, 32, 8, 128, "bf16")
    return bulk_evict_refill(name, g, seed, n_seqs, ctx, {E: 0.30, R: 0.10}, refill_chunk=refill_chunk)


def config_llama8b_32k(seed=1, n_seqs=16, refill_chunk=64):
    return config_llama8b_layer(seed, n_seqs, 32768, refill_chunk, "cfg2-32k-headline")


def config_qwen14b_budget(seed=2, n_seqs=32, n_steps=32768, budget=2048, steps_per_call=16):
    g = Geometry(1, 40, 8, 128, "bf16")
    return budgeted_decode("cfg3-qwen-14b-budget", g, seed, n_seqs, n_steps, budget, steps_per_call)


def config_gptoss(seed=3, n_seqs=128, n_layers=24, ctx_lo=4096, ctx_hi=32768, refill_chunk=64):
    g = Geometry(n_layers, 64, 8, 64, "bf16")
    rng = np.random.default_rng(seed + 1000)
    ctx = rng.integers(ctx_lo, ctx_hi + 1, size=n_seqs)
    wol = [0 if l % 2 == 0 else 128 for l in range(n_layers)]
    return bulk_evict_refill("cfg4-gpt-oss-20b", g, seed, n_seqs, ctx, {T: 0.2, E: 0.2, R: 0.2},
                             refill_chunk=refill_chunk, window_of_layer=wol)


def stress_contexts(seed=4, n_seqs=256, lo=1024, hi=65536):
    rng = np.random.default_rng(seed + 2000)
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n_seqs)).astype(np.int64)


def stress_decode(name, geom, seed, ctx_tokens, n_steps, evict_every=16, evict_frac=0.05, lowest=E):
    """Config 5: bulk-build ragged contexts, then n_steps decode steps; a step appends one token
    per sequence, and every `evict_every`-th step ends with an eviction pass that removes
    `evict_frac` of the live tokens of the lowest-importance class (seeded uniform choice, drawn
    per layer).  The decode query of the last step is the one the attention check uses."""
    rng = np.random.default_rng(seed)
    ctx = np.asarray(ctx_tokens, dtype=np.int64)
    n_seqs, L = len(ctx), geom.n_layers
    classes = []
    for s in range(n_seqs):
        c, _ = thought_classes(rng, int(ctx[s]) + n_steps)
        classes.append(c[:int(ctx[s]) + n_steps])
    ops = []
    seqs = np.arange(n_seqs, dtype=np.int32)
    ones = np.ones(n_seqs, dtype=np.int64)
    for l in range(L):
        ops.append(Append(l, seqs, np.zeros(n_seqs, np.int64), ctx.copy()))
        live_low = [np.flatnonzero(classes[s][:ctx[s]] == lowest) for s in range(n_seqs)]
        for st in range(n_steps):
            ops.append(Append(l, seqs, ctx + st, ones))
            for s in range(n_seqs):
                if classes[s][ctx[s] + st] == lowest:
                    live_low[s] = np.append(live_low[s], ctx[s] + st)
            if (st + 1) % evict_every == 0:
                es, ep = [], []
                for s in range(n_seqs):
                    n = int(round(evict_frac * len(live_low[s])))
                    if n == 0:
                        continue
                    drop = rng.choice(live_low[s], size=n, replace=False)
                    live_low[s] = np.setdiff1d(live_low[s], drop)
                    es.append(np.full(n, s, dtype=np.int32))
                    ep.append(np.sort(drop))
                if es:
                    ops.append(Evict(l, np.concatenate(es), np.concatenate(ep)))
    return Workload(name, geom, seed, n_seqs, classes, ops, tuple([0] * L), (ctx + n_steps - 1).astype(np.int32))


def config_stress(seed=4, n_seqs=256, n_layers=32, n_steps=64):
    g = Geometry(n_layers, 32, 8, 128, "bf16")
    return stress_decode("cfg5-stress-8b", g, seed, stress_contexts(seed, n_seqs), n_steps)
