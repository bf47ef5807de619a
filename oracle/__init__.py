"""CPU oracle for the ThinKV decode hot path.

TEST INFRASTRUCTURE ONLY.  This package is the plain, slow, fp64/NumPy statement of
what the hot path computes (reference group quantizer, paged-cache bookkeeping with
soft eviction and in-place slot reuse, dequantize-then-softmax decode attention).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import it.  It shares no code with the HIP path and never imports
the product package's binding; the product path never imports this package.

Pinning status (see tests/test_oracle_*.py):
  quant.quantize_groups / dequantize .... pinned (closed forms, invariants, round-trip bound)
  layout.pack_page_head ................. pinned (independent bit-by-bit unpacker, hand-written fixture)
  cache.OracleCache (bookkeeping) ....... pinned (walkthrough events of the paper's Sec. "ThinKV
                                          Walkthrough Example", brute-force dict model, invariants)
  formats (E4M3 / E2M1 / ternary codes, group quantisers with E4M3 scales) ... pinned (every code against
                                          hand-made tables and the library's 8-bit float type, rounding cases, brute force)
  attention.decode_attention ............ pinned (dense softmax on compacted tokens, Theorem 1
                                          permutation invariance, closed forms, library softmax)
"""
