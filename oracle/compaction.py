"""What a contiguous cache looks like after gather-based compaction (test infrastructure; see oracle/__init__.py).

Sec. 5.1 of the paper ("The Cost of Gather-Based Compaction"): without in-place slot reuse, every eviction is
followed by a gather that moves the surviving tokens' keys and values into a dense buffer.  The result has a
plain definition: the rows of the live tokens, in ascending logical position, and nothing else."""
import numpy as np


def live_positions(cache, seq, layer):
    """ascending logical positions of the tokens of (seq, layer) the paged cache still holds"""
    return np.array(sorted(p for p, _, _, _ in cache.live_tokens(seq, layer)), dtype=np.int64)


def compact(rows, live):
    """rows [n_tok, ...] indexed by logical position, live: ascending positions that survive -> the dense buffer"""
    out = np.empty((len(live),) + rows.shape[1:], dtype=rows.dtype)
    for i, p in enumerate(live):
        out[i] = rows[int(p)]
    return out
