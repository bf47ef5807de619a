"""Cache backends the synthetic scripts can be replayed on (test helper)."""
import numpy as np
import torch

from oracle import cache as ocache


class OracleBackend:
    device = torch.device("cpu")

    def __init__(self, cfg, store_data=True):
        self.cache = ocache.OracleCache(cfg, store_data=store_data)

    def append(self, layer, k, v, tok_seq, tok_pos, tok_class):
        return self.cache.append(layer, k.float().numpy(), v.float().numpy(), tok_seq, tok_pos, tok_class)

    def evict(self, layer, ev_seq, ev_handle):
        self.cache.evict_slots(layer, ev_seq, ev_handle)


def oracle_config(geom, max_seqs, max_pages, arena_pages):
    return ocache.OracleConfig(geom.n_layers, geom.n_q_heads, geom.n_kv_heads, geom.head_dim,
                               tuple(geom.bits_of_class), max_seqs, max_pages, tuple(arena_pages))


def arena_need(wl, slack=1.25):
    """generous per-class page counts for a workload (host-side sizing only)"""
    tot = np.zeros(3, dtype=np.int64)
    for s in range(wl.n_seqs):
        for c in range(3):
            n = int((wl.classes[s] == c).sum())
            tot[c] += (n + 15) // 16 + 2
    tot = (tot * wl.geom.n_layers * slack).astype(np.int64) + 4
    return tuple(int(x) for x in tot)


def arena_need_one(wl, s):
    """per-class page counts that hold ONE sequence in ONE layer (for an oracle that replays a sample)"""
    return tuple(int((wl.classes[s] == c).sum() + 15) // 16 + 4 for c in range(3))


def max_pages_need(wl):
    m = 1
    for s in range(wl.n_seqs):
        for c in range(3):
            m = max(m, (int((wl.classes[s] == c).sum()) + 15) // 16 + 2)
    return m
