"""thinkv_decode_attention_noalloc (the entry point for callers that cannot allocate or pass a
workspace) against thinkv_decode_attention, through the C ABI: two calls in a row, the second on a
smaller input, so that what the first call left in the library's scratch array is seen not to matter.
Both entry points run the same kernels; which wave adds which page pair to which partial row differs
from launch to launch, so the outputs agree to rounding, not bit for bit; the bar is the attention
tolerance of the other GPU tests (2e-3 max-abs on binary32 output), and the oracle is consulted too."""
import ctypes as C

import numpy as np
import pytest
import torch

import parity
from paper_2510_01290_amd import synth

pytestmark = pytest.mark.gpu


def _call(fn_name, gc, layer, q, out, lse, sid, qp, window, scale, mcp, with_ws):
    from paper_2510_01290_amd import binding as B
    lib = B.load()
    fn = getattr(lib, fn_name)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    args = [C.byref(gc.view), layer, C.c_void_p(q.data_ptr()), C.c_void_p(out.data_ptr()), C.c_void_p(lse.data_ptr()),
            C.c_void_p(sid.data_ptr()), C.c_void_p(qp.data_ptr()), int(q.shape[0]), window, C.c_float(scale),
            B._DT[q.dtype], B._DT[out.dtype], int(mcp)]
    if with_ws:
        nb = B.thinkv_decode_workspace_bytes(gc.cfg, int(q.shape[0]), int(mcp))
        ws = torch.empty(nb + 256, dtype=torch.uint8, device=gc.device)
        args += [C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel())]
    rc = fn(*args, st)
    torch.cuda.synchronize()
    return rc


def _both(gc, wl, layer, seqs):
    g = wl.geom
    dev = gc.device
    q = torch.stack([synth.query_rows(wl.seed, layer, s, 0, g, dev) for s in seqs]).contiguous()
    sid = torch.tensor(seqs, dtype=torch.int32, device=dev)
    qp = torch.from_numpy(wl.q_pos[seqs].astype(np.int32)).to(dev)
    mcp = int(gc.n_pages[:, layer].sum(-1).max().item())
    res = {}
    for name, with_ws in (("thinkv_decode_attention", True), ("thinkv_decode_attention_noalloc", False)):
        out = torch.full(q.shape, 7.0, dtype=torch.float32, device=dev)
        lse = torch.full((len(seqs), g.n_q_heads), 7.0, dtype=torch.float32, device=dev)
        rc = _call(name, gc, layer, q, out, lse, sid, qp, wl.window_of_layer[layer], g.head_dim ** -0.5, mcp, with_ws)
        assert rc == 0, (name, rc)
        res[name] = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
    return res


def test_noalloc_entry_point_matches_the_workspace_one_twice_in_a_row():
    from paper_2510_01290_amd import binding as B
    print("no-alloc decode attention against the workspace entry point: a larger call, then a smaller one", flush=True)
    geom = synth.Geometry(2, 32, 8, 128, "bf16", (8, 2, 4))
    wl = synth.bulk_evict_refill("noalloc", geom, 77, 4, np.array([3000, 900, 5000, 40]), {synth.E: 0.3, synth.R: 0.1}, refill_chunk=16,
                                 window_of_layer=(0, 128))
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    ob = parity.make_oracle(wl)
    synth.ScriptRunner(wl, ob).run()
    torch.cuda.synchronize()
    for layer, seqs in ((0, [0, 1, 2, 3]), (0, [3, 1]), (1, [2, 0, 1]), (1, [3])):      # each second call is the smaller one
        res = _both(gc, wl, layer, seqs)
        a, la = res["thinkv_decode_attention"]
        b, lb = res["thinkv_decode_attention_noalloc"]
        ref, ref_lse = parity.oracle_attention(ob.cache, wl, layer, seqs, seqs)
        assert np.abs(b - a).max() <= parity.TOL and np.abs(b - ref).max() <= parity.TOL, (layer, seqs, np.abs(b - a).max(), np.abs(b - ref).max())
        fin = np.isfinite(ref_lse)
        assert np.array_equal(np.isfinite(lb), fin) and np.abs(lb[fin] - ref_lse[fin]).max() <= 1e-3 and np.abs(lb[fin] - la[fin]).max() <= 1e-3
        print("  layer", layer, "sequences", seqs, "max |noalloc - workspace|", float(np.abs(b - a).max()), "max |noalloc - oracle|", float(np.abs(b - ref).max()), flush=True)
    assert int(gc.dev_status.abs().sum().item()) == 0
    # a launch whose partial rows do not fit the scratch array is refused, and nothing is launched
    big = B.make_config(1, 64, 8, 128, (8, 2, 4), 4096, 8192)
    need = B.thinkv_decode_workspace_bytes(big, 4096, 8192)
    assert need > B.NOALLOC_SCRATCH_BYTES
    v = B.View()
    C.memmove(C.byref(v), C.byref(gc.view), C.sizeof(B.View))
    v.cfg = big
    rc = B.load().thinkv_decode_attention_noalloc(C.byref(v), 0, None, None, None, None, None, 4096, 0, C.c_float(0.1), 1, 2, 8192, None)
    assert rc == 4, rc
