"""The gather-compaction contrast kernel (thinkv_gather_rows) against the oracle's statement of compaction: the
dense buffer is the rows of the tokens the paged cache still holds, in ascending position, bit for bit."""
import ctypes as C

import numpy as np
import pytest
import torch

import parity
from oracle import compaction
from paper_2510_01290_amd import synth

pytestmark = pytest.mark.gpu


def test_gather_compaction_equals_the_oracles_live_rows():
    from paper_2510_01290_amd import binding as B
    print("gather-based compaction of a contiguous 16-bit cache: survivors of three sequences, K and V", flush=True)
    geom = synth.Geometry(1, 32, 8, 128, "bf16", (8, 2, 4))
    ctx = np.array([5000, 333, 16])
    wl = synth.bulk_evict_refill("gather", geom, 9, 3, ctx, {synth.E: 0.3, synth.R: 0.1, synth.T: 0.05}, refill=0)
    ob = parity.make_oracle(wl, store_data=False)
    synth.ScriptRunner(wl, ob).run()
    dev = torch.device("cuda:0")
    for kind in (0, 1):
        # the contiguous cache: every sequence's rows one after the other, a row = one token's K (or V) of all kv-heads
        rows = torch.cat([synth.kv_rows(wl.seed, 0, s, kind, 0, int(ctx[s]), geom, dev).reshape(int(ctx[s]), -1) for s in range(3)]).contiguous()
        base = np.r_[0, np.cumsum(ctx)]
        live = np.concatenate([base[s] + compaction.live_positions(ob.cache, s, 0) for s in range(3)])
        assert 0 < len(live) < rows.shape[0]
        idx = torch.from_numpy(live.astype(np.int32)).to(dev)
        dst = torch.full((len(live), rows.shape[1]), 7.0, dtype=rows.dtype, device=dev)
        B.thinkv_gather_rows(rows, dst, idx)
        torch.cuda.synchronize()
        want = compaction.compact(rows.view(torch.int16).cpu().numpy(), live)
        assert np.array_equal(dst.view(torch.int16).cpu().numpy(), want)
    # rows of 16 bytes, a single row, no rows; bad arguments are refused on the host
    small = torch.arange(64 * 8, dtype=torch.int16, device=dev).reshape(64, 8)
    pick = torch.tensor([63, 0, 5, 5, 17], dtype=torch.int32, device=dev)
    out = torch.zeros((5, 8), dtype=torch.int16, device=dev)
    B.thinkv_gather_rows(small, out, pick)
    torch.cuda.synchronize()
    assert torch.equal(out, small[pick.long()])
    lib = B.load()
    assert lib.thinkv_gather_rows(C.c_void_p(small.data_ptr()), C.c_void_p(out.data_ptr()), C.c_void_p(pick.data_ptr()), 0, 16, None) == 0
    assert lib.thinkv_gather_rows(C.c_void_p(small.data_ptr()), C.c_void_p(out.data_ptr()), C.c_void_p(pick.data_ptr()), 5, 24, None) == 1
    assert lib.thinkv_gather_rows(None, C.c_void_p(out.data_ptr()), C.c_void_p(pick.data_ptr()), 5, 16, None) == 1
