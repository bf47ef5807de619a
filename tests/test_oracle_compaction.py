"""The oracle's statement of gather-based compaction (oracle/compaction.py): the dense buffer holds the rows of the
live tokens in ascending position.  Pinned against the script itself (what was appended minus what was evicted) and
against the library's boolean-mask indexing."""
import numpy as np

import parity
from oracle import compaction
from paper_2510_01290_amd import synth


def test_compaction_is_the_live_rows_in_order():
    geom = synth.Geometry(2, 8, 2, 64, "f16", (8, 2, 4))
    wl = synth.bulk_evict_refill("compact", geom, 5, 2, np.array([300, 77]), {synth.E: 0.5, synth.T: 0.2}, refill=40, refill_chunk=8)
    ob = parity.make_oracle(wl, store_data=False)
    synth.ScriptRunner(wl, ob).run()
    for l in range(2):
        for s in range(2):
            alive = np.zeros(len(wl.classes[s]), bool)
            for op in wl.ops:
                if op.layer != l:
                    continue
                if isinstance(op, synth.Append):
                    i = list(op.seqs).index(s)
                    alive[op.t0[i]:op.t0[i] + op.cnt[i]] = True
                else:
                    alive[op.pos[op.seqs == s]] = False
            live = compaction.live_positions(ob.cache, s, l)
            assert np.array_equal(live, np.flatnonzero(alive))
            rows = np.arange(len(alive) * 6, dtype=np.uint16).reshape(len(alive), 6)
            assert np.array_equal(compaction.compact(rows, live), rows[alive])
    assert compaction.compact(np.zeros((4, 3)), np.zeros(0, np.int64)).shape == (0, 3)
