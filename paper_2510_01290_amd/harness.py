"""Driving the HIP cache from a synthetic workload script (bench.py, the GPU tests): host-side
sizing of the arenas and tables, construction of a device cache for a workload, and the backend
object `synth.ScriptRunner` replays a script on.  Argument plumbing only; nothing here touches the
CPU oracle, and none of the method's arithmetic lives here."""
import numpy as np
import torch


def arena_need(wl, slack=1.25):
    """generous per-type page counts for a workload (host-side sizing only)"""
    tot = np.zeros(3, dtype=np.int64)
    for s in range(wl.n_seqs):
        for c in range(3):
            n = int((wl.classes[s] == c).sum())
            tot[c] += (n + 15) // 16 + 2
    tot = (tot * wl.geom.n_layers * slack).astype(np.int64) + 4
    return tuple(int(x) for x in tot)


def arena_need_one(wl, s):
    """per-type page counts that hold ONE sequence in ONE layer (for a replay of a sample)"""
    return tuple(int((wl.classes[s] == c).sum() + 15) // 16 + 4 for c in range(3))


def max_pages_need(wl):
    m = 1
    for s in range(wl.n_seqs):
        for c in range(3):
            m = max(m, (int((wl.classes[s] == c).sum()) + 15) // 16 + 2)
    return m


class GpuBackend:
    """`synth.ScriptRunner` backend that drives a `binding.Cache` through the C ABI"""

    def __init__(self, cache):
        self.cache = cache
        self.device = cache.device

    def append(self, layer, k, v, tok_seq, tok_pos, tok_class):
        from . import binding as B
        d = self.device
        ts = torch.from_numpy(np.ascontiguousarray(tok_seq, dtype=np.int32)).to(d)
        tp = torch.from_numpy(np.ascontiguousarray(tok_pos, dtype=np.int32)).to(d)
        tc = torch.from_numpy(np.ascontiguousarray(tok_class, dtype=np.uint8)).to(d)
        h = torch.empty(len(tok_seq), dtype=torch.int32, device=d)
        B.thinkv_append_quantized(self.cache, layer, k.contiguous(), v.contiguous(), ts, tp, tc, h)
        return h.cpu().numpy()

    def evict(self, layer, ev_seq, ev_handle):
        from . import binding as B
        d = self.device
        B.thinkv_evict(self.cache, layer, torch.from_numpy(np.ascontiguousarray(ev_seq, dtype=np.int32)).to(d),
                       torch.from_numpy(np.ascontiguousarray(ev_handle, dtype=np.int32)).to(d))


def make_gpu_cache(wl, max_seqs=None, arena_pages=None, max_pages=None, device="cuda:0"):
    from . import binding as B
    g = wl.geom
    return B.Cache(g.n_layers, g.n_q_heads, g.n_kv_heads, g.head_dim, g.bits_of_class,
                   max_seqs or wl.n_seqs, max_pages or max_pages_need(wl),
                   arena_pages or arena_need(wl), device=device,
                   fmt=B.FMT_FP if getattr(g, "fmt", "int") == "fp" else B.FMT_INT, fp8_scale=tuple(getattr(g, "fp8_scale", (1.0, 1.0))))
