"""The attention-sparsity statistic of a decode step: HIP path against the oracle (needs an MI355X).

The statistic is a count decided by a floating-point comparison (pooled score against the row
maximum less ln 100).  The device compares binary32 scores, the oracle binary64 ones, so an
entry within rounding of the boundary may fall on either side: the oracle's count is taken
with the boundary moved by -DELTA and +DELTA (score units) and the device value has to lie
between the two; most cases have no entry that close, and then the two bounds coincide and
the comparison is exact up to the binary32 division."""
import numpy as np
import pytest
import torch

import parity
from oracle import attention as oattn
from oracle import sparsity as osp
from paper_2510_01290_amd import synth

pytestmark = pytest.mark.gpu

DELTA = 5e-4
LN100 = np.log(100.0)


def _say(msg):
    print(msg, flush=True)


def _oracle_bounds(oc, wl, layer, so, sw):
    g = wl.geom
    q = synth.query_rows(wl.seed, layer, sw, 0, g, torch.device("cpu")).float().numpy().astype(np.float64)
    _, k, _ = oattn.gather_live(oc, so, layer, int(wl.q_pos[sw]), wl.window_of_layer[layer])
    pooled = osp.pooled_scores(q, k, g.head_dim ** -0.5)
    lo, hi, mid = [], [], []
    for h in range(pooled.shape[0]):
        n = pooled.shape[1]
        if n == 0:
            lo.append(0.0), hi.append(0.0), mid.append(0.0)
            continue
        cut = pooled[h].max() - LN100
        lo.append(np.count_nonzero(pooled[h] < cut - DELTA) / n)
        hi.append(np.count_nonzero(pooled[h] < cut + DELTA) / n)
        mid.append(osp.row_sparsity(pooled[h]))
    return float(np.mean(lo)), float(np.mean(hi)), float(np.mean(mid))


def _gpu(gc, wl, layer, out_dtype=torch.float32, max_ctx_pages=None):
    from paper_2510_01290_amd import binding as B
    g = wl.geom
    seqs = list(range(wl.n_seqs))
    q = torch.stack([synth.query_rows(wl.seed, layer, s, 0, g, gc.device) for s in seqs]).contiguous()
    out = torch.empty(q.shape, dtype=out_dtype, device=gc.device)
    lse = torch.empty((len(seqs), g.n_q_heads), dtype=torch.float32, device=gc.device)
    sp = torch.full((len(seqs),), -1.0, dtype=torch.float32, device=gc.device)
    sid = torch.tensor(seqs, dtype=torch.int32, device=gc.device)
    qp = torch.from_numpy(wl.q_pos[seqs].astype(np.int32)).to(gc.device)
    if max_ctx_pages is None:
        max_ctx_pages = int(gc.n_pages[:, layer].sum(-1).max().item())
    B.thinkv_decode_attention_sparsity(gc, layer, q, out, lse, sp, sid, qp, wl.window_of_layer[layer], g.head_dim ** -0.5, max_ctx_pages)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64), sp.cpu().numpy().astype(np.float64)


def _run(wl, sample=None):
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    torch.cuda.synchronize()
    assert int(gc.dev_status.abs().sum().item()) == 0
    pairs = [(s, l) for s in range(wl.n_seqs) for l in range(wl.geom.n_layers)] if sample is None else sample
    caches = {}
    if sample is None:
        ob = parity.make_oracle(wl)
        synth.ScriptRunner(wl, ob).run()
        for s, l in pairs:
            caches[(s, l)] = ob.cache
    else:
        for s, l in pairs:
            ob = parity.make_oracle(wl, max_seqs=wl.n_seqs, arena_pages=parity.backends.arena_need_one(wl, s))
            synth.ScriptRunner(wl, ob, layers=[l], seqs=[s]).run()
            caches[(s, l)] = ob.cache
    exact = 0
    worst = 0.0
    for l in sorted({l for _, l in pairs}):
        got, lse, sp = _gpu(gc, wl, l)
        plain, plain_lse = parity.gpu_attention(gc, wl, None, l, torch.float32, "fast")
        assert np.abs(got - plain).max() <= 1e-4 and np.array_equal(np.isfinite(lse), np.isfinite(plain_lse))   # same attention as the plain call (the split of the work differs from run to run)
        assert np.all((sp >= 0.0) & (sp <= 1.0))
        for s, l2 in pairs:
            if l2 != l:
                continue
            oc = caches[(s, l)]
            ref, ref_lse = parity.oracle_attention(oc, wl, l, [s], [s])
            assert np.abs(got[s] - ref[0]).max() <= parity.TOL
            lo, hi, mid = _oracle_bounds(oc, wl, l, s, s)
            assert lo - 1e-6 <= sp[s] <= hi + 1e-6, ("sparsity", s, l, sp[s], lo, hi)
            exact += int(abs(sp[s] - mid) <= 1e-6)
            worst = max(worst, abs(sp[s] - mid))
    return {"workload": wl.name, "pairs": len(pairs), "equal_to_oracle": exact, "max_abs_diff": worst}


@pytest.mark.parametrize("bits", [(8, 2, 4), (2, 4, 8)], ids=["T8E2R4", "paper-R8E4T2"])
def test_sparsity_config1_tiny(bits):
    _say(f"sparsity statistic, config 1 tiny, bits(T,E,R)={bits}")
    _say(_run(synth.config_tiny(0, bits)))


@pytest.mark.parametrize("D,dtype,G", [(128, "bf16", 4), (64, "bf16", 8), (128, "f16", 5), (64, "f16", 1)])
def test_sparsity_ragged_multi_sequence(D, dtype, G):
    _say(f"sparsity statistic, ragged multi-seq D={D} {dtype} G={G}")
    geom = synth.Geometry(2, 2 * G, 2, D, dtype, (8, 2, 4))
    wl = synth.bulk_evict_refill("ragged", geom, 5, 4, np.array([300, 17, 1000, 1]), {synth.E: 0.3, synth.R: 0.1, synth.T: 0.05},
                                 refill_chunk=3)
    _say(_run(wl))


@pytest.mark.parametrize("D,G", [(128, 4), (64, 8)])
def test_sparsity_in_the_papers_formats(D, G):
    _say(f"sparsity statistic over a cache in FP8 / NVFP4 / ternary, D={D} G={G}, layer 1 with a window")
    geom = synth.Geometry(2, 2 * G, 2, D, "bf16", (2, 4, 8), "fp", (0.05, 0.05))
    wl = synth.bulk_evict_refill("ragged-fp", geom, 7, 3, np.array([500, 33, 1200]), {synth.E: 0.3, synth.R: 0.1}, refill_chunk=4,
                                 window_of_layer=[0, 128])
    _say(_run(wl))


def test_sparsity_window_and_empty():
    _say("sparsity statistic on a sliding-window layer, and with nothing visible")
    geom = synth.Geometry(2, 16, 2, 64, "bf16", (8, 2, 4))
    wl = synth.bulk_evict_refill("window", geom, 9, 3, np.array([700, 90, 2000]), {synth.T: 0.2, synth.E: 0.2, synth.R: 0.2},
                                 refill_chunk=5, window_of_layer=[0, 128])
    _say(_run(wl))
    # queries far beyond every stored position: the window is empty, the statistic 0
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    wl.q_pos = wl.q_pos + 100000
    got, lse, sp = _gpu(gc, wl, 1)
    assert not got.any() and np.all(np.isneginf(lse)) and not sp.any()


def test_sparsity_budgeted_decode_scrambled_slots():
    _say("sparsity statistic after budgeted decode (sparse, scrambled pages)")
    geom = synth.Geometry(1, 10, 2, 128, "bf16", (8, 2, 4))
    wl = synth.budgeted_decode("budget-small", geom, 2, 3, 3000, 512, steps_per_call=8)
    _say(_run(wl))


def test_sparsity_bench_workload_sampled():
    """the bench workload (16 x 32,768 tokens), whole-batch launch, two sequences replayed by the oracle"""
    _say("sparsity statistic at the bench size")
    wl = synth.config_llama8b_32k(seed=1, n_seqs=16, refill_chunk=64)
    _say(_run(wl, sample=[(2, 0), (13, 0)]))


def test_sparsity_context_bound_too_small_is_safe():
    _say("a context bound below the true page count: counted over the first pages only, nothing written out of bounds")
    geom = synth.Geometry(1, 8, 2, 64, "f16", (8, 2, 4))
    wl = synth.bulk_evict_refill("short-bound", geom, 11, 2, np.array([900, 400]), {synth.E: 0.2}, refill_chunk=7)
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    true_pages = int(gc.n_pages[:, 0].sum(-1).max().item())
    from paper_2510_01290_amd import binding as B
    nb = B.load().thinkv_decode_sparsity_workspace_bytes(__import__("ctypes").byref(gc.cfg), 2, true_pages // 2)
    guard = gc.workspace(nb + 4096)
    guard.fill_(0x5A)
    got, lse, sp = _gpu(gc, wl, 0, max_ctx_pages=true_pages // 2)
    assert np.all((sp >= 0.0) & (sp <= 1.0))
    assert bool((guard[nb:nb + 4096] == 0x5A).all().item()), "wrote past the workspace it asked for"
