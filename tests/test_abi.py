"""The C-ABI library loads, exports every symbol the header declares, and its host-side
entry points behave without a GPU (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2510_01290_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    from paper_2510_01290_amd import binding
    hdr = open(os.path.join(ROOT, "include", "thinkv.h")).read()
    declared = set(re.findall(r"\b(thinkv_[a-z_]+)\s*\(", hdr))
    declared -= {"thinkv_status"}           # typedef names never followed by '(' anyway
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_layout_queries_match_the_stated_formula(lib):
    from paper_2510_01290_amd import binding as B
    for D in (64, 128):
        cfg = B.make_config(1, 8, 2, D, (8, 2, 4), 4, 16)
        for bits in (2, 4, 8):
            assert B.thinkv_block_bytes(cfg, bits) == 16 * 2 * (D * bits // 8 + (D // 32) * 4)
            assert B.thinkv_page_bytes(cfg, bits) == 2 * B.thinkv_block_bytes(cfg, bits)
        assert B.thinkv_block_bytes(cfg, 3) == 0
    bad = B.make_config(1, 8, 2, 96, (8, 2, 4), 4, 16)
    assert B.thinkv_block_bytes(bad, 4) == 0
    assert B.thinkv_append_workspace_bytes(cfg, 100) > 0
    assert B.thinkv_decode_workspace_bytes(cfg, 3, 100) >= 3 * 8 * (128 + 2) * 4


def test_host_side_argument_errors(lib):
    from paper_2510_01290_amd import binding as B
    assert lib.thinkv_init_view(None, None) == 1
    v = B.View()
    v.cfg = B.make_config(1, 8, 2, 128, (8, 2, 4), 4, 16)
    assert lib.thinkv_init_view(C.byref(v), None) == 1            # null device pointers
    v.cfg = B.make_config(1, 8, 3, 128, (8, 2, 4), 4, 16)
    assert lib.thinkv_init_view(C.byref(v), None) == 2            # 8 heads do not group over 3
    v.cfg = B.make_config(1, 8, 2, 128, (8, 3, 4), 4, 16)
    assert lib.thinkv_evict(C.byref(v), 0, None, None, 0, None) == 2
    assert lib.thinkv_status_string(4) == b"workspace too small"
