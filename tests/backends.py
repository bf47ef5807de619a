"""Cache backends the synthetic scripts can be replayed on (test helper)."""
import numpy as np
import torch

from oracle import cache as ocache
from paper_2510_01290_amd.harness import arena_need, arena_need_one, max_pages_need  # noqa: F401  (sizing, shared with the device side)


class OracleBackend:
    device = torch.device("cpu")

    def __init__(self, cfg, store_data=True):
        self.cache = ocache.OracleCache(cfg, store_data=store_data)
        self.needs_data = store_data

    def append(self, layer, k, v, tok_seq, tok_pos, tok_class):
        if not self.needs_data:
            return self.cache.append(layer, None, None, tok_seq, tok_pos, tok_class)
        return self.cache.append(layer, k.float().numpy(), v.float().numpy(), tok_seq, tok_pos, tok_class)

    def evict(self, layer, ev_seq, ev_handle):
        self.cache.evict_slots(layer, ev_seq, ev_handle)


def oracle_config(geom, max_seqs, max_pages, arena_pages):
    return ocache.OracleConfig(geom.n_layers, geom.n_q_heads, geom.n_kv_heads, geom.head_dim,
                               tuple(geom.bits_of_class), max_seqs, max_pages, tuple(arena_pages),
                               fmt=getattr(geom, "fmt", "int"), fp8_scale=tuple(getattr(geom, "fp8_scale", (1.0, 1.0))))
