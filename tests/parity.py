"""GPU-vs-oracle parity harness (test helper; also used by __graft_entry__.smoke and bench.py's
cpu_baseline leg).  The same seeded script is replayed on the HIP cache and on the CPU oracle;
bookkeeping and packed bytes are compared bit for bit, attention within the stated tolerance."""
import time
from dataclasses import dataclass, field

import numpy as np
import torch

from oracle import attention as oattn
from oracle import cache as ocache
from paper_2510_01290_amd import synth
from paper_2510_01290_amd.harness import GpuBackend, make_gpu_cache  # noqa: F401

import backends

TOL = 2e-3          # max-abs error of the attention output against the binary64 oracle (binary32 out)


def make_oracle(wl, max_seqs=None, arena_pages=None, max_pages=None, store_data=True):
    cfg = backends.oracle_config(wl.geom, max_seqs or wl.n_seqs, max_pages or backends.max_pages_need(wl),
                                 arena_pages or backends.arena_need(wl))
    return backends.OracleBackend(cfg, store_data=store_data)


# ------------------------------------------------------------------------- comparisons
def gpu_tables(gc):
    """host copies of the device bookkeeping"""
    t = dict(table=gc.block_table.cpu().numpy(), n_pages=gc.n_pages.cpu().numpy(), n_live=gc.n_live.cpu().numpy(),
             status=gc.dev_status.cpu().numpy().view(np.uint32), free_top=gc.free_top.cpu().numpy())
    t["filled"] = [x.cpu().numpy() for x in gc.page_filled]
    t["mask"] = gc.slot_mask.cpu().numpy().view(np.uint32)      # [seq][layer][type][list position]
    t["slot_pos"] = [x.cpu().numpy() for x in gc.slot_pos]
    t["pos_max"] = [x.cpu().numpy() for x in gc.page_pos_max]
    t["free_stack"] = [x.cpu().numpy() for x in gc.free_stack]
    return t


def compare_bookkeeping_full(oc, gc):
    """every table, mask, counter and the free pools, bit for bit (same physical page ids)"""
    t = gpu_tables(gc)
    assert np.array_equal(t["n_pages"], oc.n_pages), "n_pages"
    assert np.array_equal(t["n_live"], oc.n_live), "n_live"
    assert np.array_equal(t["status"], oc.status), ("dev_status", t["status"], oc.status)
    assert np.array_equal(t["free_top"], oc.free_top), "free_top"
    S, L = oc.n_pages.shape[:2]
    for s in range(S):
        for l in range(L):
            for c in range(3):
                n = int(oc.n_pages[s, l, c])
                assert np.array_equal(t["table"][s, l, c, :n], oc.table[s, l, c, :n]), ("block_table", s, l, c)
                pages = oc.table[s, l, c, :n]
                assert np.array_equal(t["mask"][s, l, c, :n] & 0xFFFF, oc.valid[c][pages]), ("live bits", s, l, c)
                assert np.array_equal(t["mask"][s, l, c, :n] >> 16, oc.evict[c][pages]), ("evict bits", s, l, c)
    for c in range(3):
        n = int(oc.cfg.arena_pages[c])
        top = int(oc.free_top[c])
        assert np.array_equal(t["free_stack"][c][:top], oc.free_stack[c][:top]), "free_stack"
        used = np.setdiff1d(np.arange(n), oc.free_stack[c][:top])
        assert np.array_equal(t["filled"][c][used], oc.filled[c][used]), "filled"
        assert np.array_equal(t["slot_pos"][c][used], oc.slot_pos[c][used]), "slot_pos"
        # the window kernel's page filter: never below any position the page holds, -1 on untouched pages
        assert (t["pos_max"][c][used] >= oc.slot_pos[c][used].max(axis=1)).all(), "page_pos_max below a stored position"
        free = oc.free_stack[c][:top]
        assert (t["pos_max"][c][free] == -1).all(), "page_pos_max set on a page never handed out"


def compare_sequences(oc, gc, pairs, check_bytes=True):
    """per (oracle seq, gpu seq, layer): page lists compared page by page through the tables, so it
    also works when the oracle replayed only a sample of the sequences (different physical ids)"""
    t = gpu_tables(gc)
    for so, sg, l in pairs:
        assert np.array_equal(t["n_pages"][sg, l], oc.n_pages[so, l]), ("n_pages", sg, l)
        assert t["n_live"][sg, l] == oc.n_live[so, l], ("n_live", sg, l)
        for c in range(3):
            n = int(oc.n_pages[so, l, c])
            po = oc.table[so, l, c, :n]
            pg = t["table"][sg, l, c, :n]
            assert np.array_equal(t["filled"][c][pg], oc.filled[c][po]), ("filled", sg, l, c)
            assert np.array_equal(t["mask"][sg, l, c, :n] & 0xFFFF, oc.valid[c][po]), ("live bits", sg, l, c)
            assert np.array_equal(t["mask"][sg, l, c, :n] >> 16, oc.evict[c][po]), ("evict bits", sg, l, c)
            assert np.array_equal(t["slot_pos"][c][pg], oc.slot_pos[c][po]), ("slot_pos", sg, l, c)
            if n:
                assert (t["pos_max"][c][pg] >= oc.slot_pos[c][po].max(axis=1)).all(), ("page_pos_max", sg, l, c)
            if check_bytes and n:
                pb = gc.page_bytes[c]
                idx = torch.from_numpy(pg.astype(np.int64)).to(gc.device)
                img_g = gc.arena[c].view(-1, pb)[idx].cpu().numpy()
                img_o = oc.arena_image_pages(c, po)
                assert np.array_equal(img_g, img_o), ("page bytes", sg, l, c)


def gpu_attention(gc, wl, runner, layer, out_dtype=torch.float32, variant="fast", seqs=None, max_ctx_pages=None):
    from paper_2510_01290_amd import binding as B
    g = wl.geom
    seqs = list(range(wl.n_seqs)) if seqs is None else list(seqs)
    q = torch.stack([synth.query_rows(wl.seed, layer, s, 0, g, gc.device) for s in seqs]).contiguous()
    out = torch.empty(q.shape, dtype=out_dtype, device=gc.device)
    lse = torch.empty((len(seqs), g.n_q_heads), dtype=torch.float32, device=gc.device)
    sid = torch.tensor(seqs, dtype=torch.int32, device=gc.device)
    qp = torch.from_numpy(wl.q_pos[seqs].astype(np.int32)).to(gc.device)
    if max_ctx_pages is None:
        max_ctx_pages = int(gc.n_pages[:, layer].sum(-1).max().item())
    fn = B.thinkv_decode_attention if variant == "fast" else B.thinkv_decode_attention_valu
    fn(gc, layer, q, out, lse, sid, qp, wl.window_of_layer[layer], g.head_dim ** -0.5, max_ctx_pages)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


def oracle_attention(oc, wl, layer, seqs_oracle, seqs_workload):
    g = wl.geom
    q = torch.stack([synth.query_rows(wl.seed, layer, s, 0, g, torch.device("cpu")) for s in seqs_workload])
    return oattn.decode_attention(oc, layer, q.float().numpy().astype(np.float64), seqs_oracle,
                                  wl.q_pos[list(seqs_workload)], wl.window_of_layer[layer], g.head_dim ** -0.5)


def half_ulp(ref, dtype):
    """half a unit in the last place of `dtype` at |ref| (rounding allowance for 16-bit outputs)"""
    mant = {torch.float16: 10, torch.bfloat16: 7}[dtype]
    e = np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -14)))
    return 2.0 ** (e - mant - 1)


# ------------------------------------------------------------------------------- cases
@dataclass
class Case:
    wl: object
    sample: list = None          # (seq, layer) pairs the oracle replays; None = everything
    variants: tuple = ("fast", "valu")
    cross_check_all: bool = False   # sampled cases: also compare the two device kernels on every sequence
    full_tables: bool = False       # sampled cases: also replay EVERY sequence and layer on an oracle that keeps the tables
                                    # only (no K/V data) and compare every handle, table, mask, counter and free pool


def case_tiny(seed=0, bits=(8, 2, 4)):
    return Case(synth.config_tiny(seed, bits))


def _check_rows(worst, got, lse, ref, ref_lse, dt, variant, where):
    err = np.abs(got - ref)
    allow = TOL + (half_ulp(ref, dt) if dt != torch.float32 else 0.0)
    key = f"attn_max_abs_err_{'f32' if dt == torch.float32 else str(dt).split('.')[-1]}" + ("" if variant == "fast" else "_valu")
    worst[key] = max(worst.get(key, 0.0), float(err.max()))
    assert np.all(err <= allow), (key, where, float(err.max()))
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isfinite(lse), fin), ("lse finiteness", where)
    assert np.all(np.abs(lse[fin] - ref_lse[fin]) <= 1e-3), ("lse", where, float(np.abs(lse[fin] - ref_lse[fin]).max()))


def run_case(case, check_bytes=True, out_dtypes=(torch.float32,)):
    """Replays the workload on the device; replays all of it (or the sampled (sequence, layer)
    pairs) on the oracle; compares handles, bookkeeping, page bytes and attention.  Attention is
    always launched for the whole batch, as the benchmark launches it; in sampled cases the rows
    of the sampled sequences are the ones compared with the oracle."""
    wl = case.wl
    gc = make_gpu_cache(wl)
    gr = synth.ScriptRunner(wl, GpuBackend(gc)).run()
    torch.cuda.synchronize()
    assert int(gc.dev_status.abs().sum().item()) == 0, "device flags set while replaying the workload"
    res = {"workload": wl.name}
    all_seqs = list(range(wl.n_seqs))
    per_layer = {}          # layer -> list of (workload seq, oracle seq, oracle cache)
    if case.sample is None:
        ob = make_oracle(wl)
        orr = synth.ScriptRunner(wl, ob).run()
        for key in gr.handle:
            assert np.array_equal(gr.handle[key], orr.handle[key]), ("handles", key)
        compare_bookkeeping_full(ob.cache, gc)
        pairs = [(s, s, l) for s in all_seqs for l in range(wl.geom.n_layers)]
        compare_sequences(ob.cache, gc, pairs, check_bytes)
        for l in range(wl.geom.n_layers):
            per_layer[l] = [(s, s, ob.cache) for s in all_seqs]
    else:
        for s, l in case.sample:
            ob = make_oracle(wl, max_seqs=wl.n_seqs, arena_pages=backends.arena_need_one(wl, s))
            orr = synth.ScriptRunner(wl, ob, layers=[l], seqs=[s]).run()
            assert np.array_equal(gr.handle[(l, s)], orr.handle[(l, s)]), ("handles", s, l)
            compare_sequences(ob.cache, gc, [(s, s, l)], check_bytes)
            per_layer.setdefault(l, []).append((s, s, ob.cache))
        if case.full_tables:
            t0 = time.time()
            ob = make_oracle(wl, store_data=False)
            orr = synth.ScriptRunner(wl, ob).run()
            for key in gr.handle:
                assert np.array_equal(gr.handle[key], orr.handle[key]), ("handles", key)
            compare_bookkeeping_full(ob.cache, gc)
            res["all_tables_compared_seconds"] = round(time.time() - t0, 1)
    worst = {}
    for l, rows in per_layer.items():
        refs = {}
        for sw, so, oc in rows:
            r, rl = oracle_attention(oc, wl, l, [so], [sw])
            refs[sw] = (r[0], rl[0])
        outs = {}
        for variant in case.variants:
            for dt in out_dtypes:
                got, lse = gpu_attention(gc, wl, gr, l, dt, variant, seqs=all_seqs)
                outs[(variant, dt)] = got
                for sw in refs:
                    _check_rows(worst, got[sw], lse[sw], refs[sw][0], refs[sw][1], dt, variant, (l, sw))
        if case.cross_check_all and ("fast", torch.float32) in outs and ("valu", torch.float32) in outs:
            d = float(np.abs(outs[("fast", torch.float32)] - outs[("valu", torch.float32)]).max())
            worst["fast_vs_valu_all_rows"] = max(worst.get("fast_vs_valu_all_rows", 0.0), d)
            assert d <= TOL, ("fast vs valu kernel", l, d)
    res.update(worst)
    return res
