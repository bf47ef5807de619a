"""The five benchmark configurations at (or near) full size (needs an MI355X).  Attention is launched for
the whole batch, as the benchmark launches it.  The oracle replays at least eight sampled (sequence, layer)
pairs with their data (handles, tables, masks and page bytes bit for bit; attention rows to 2e-3), replays
EVERY sequence and layer without data for the bookkeeping (every handle, table, mask, counter and free pool
bit for bit), and the two device kernels are cross-checked on every row."""
import numpy as np
import pytest
import torch

import parity
from paper_2510_01290_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _run(wl, sample, out_dtypes=(torch.float32,)):
    _say(f"{wl.name}: {wl.n_seqs} sequences, {wl.geom.n_layers} layer(s), sample {sample}")
    assert len(sample) >= 8
    res = parity.run_case(parity.Case(wl, sample=sample, cross_check_all=True, full_tables=True), out_dtypes=out_dtypes)
    _say(res)
    return res


def test_config2_llama8b_layer_8k():
    """config 2 as stated: batch 16, 8,192 cached tokens per sequence"""
    _run(synth.config_llama8b_layer(seed=1, n_seqs=16, ctx=8192, refill_chunk=64), [(s, 0) for s in (0, 2, 3, 5, 8, 11, 12, 15)],
         out_dtypes=(torch.float32, torch.bfloat16))


def test_config2_headline_32k_as_benchmarked():
    """the bench workload: batch 16, 32,768 live tokens per sequence"""
    _run(synth.config_llama8b_32k(seed=1, n_seqs=16, refill_chunk=64), [(s, 0) for s in (0, 1, 4, 6, 9, 10, 13, 14)])


def test_config2_headline_32k_in_the_papers_formats():
    """the bench workload with the cache in the paper's own formats (FP8-E4M3 / NVFP4 / ternary, the paper's map R8 / E4 / T2)"""
    wl = synth.config_llama8b_32k(seed=1, n_seqs=16, refill_chunk=64)
    wl.geom.bits_of_class, wl.geom.fmt, wl.geom.fp8_scale = (2, 4, 8), "fp", (0.05, 0.05)
    _run(wl, [(s, 0) for s in (0, 2, 5, 7, 8, 11, 12, 15)])


def test_config3_qwen14b_budgeted_decode():
    """config 3 at full size: 32 trajectories of 32,768 decode appends under a 2,048-token budget (G = 5)"""
    res = _run(synth.config_qwen14b_budget(), [(s, 0) for s in (0, 5, 9, 14, 18, 23, 27, 30)])
    assert "attn_max_abs_err_f32" in res


def test_config4_gptoss_full_and_window_layers():
    """config 4 with 4 of its 24 layers (layers are independent; 0 and 2 full attention, 1 and 3 window 128):
    batch 128, contexts uniform in 4k..32k, G = 8, head_dim 64"""
    wl = synth.config_gptoss(n_layers=4)
    _run(wl, [(17, 0), (90, 0), (100, 1), (41, 1), (63, 2), (127, 2), (5, 3), (72, 3)])


def test_config5_stress_ragged_decode_steps():
    """config 5 with 2 of its 32 layers (layers are independent: fewer layers shorten the test without changing any
    shape a kernel sees) and all 64 steps (four eviction passes): batch 256, contexts log-uniform in 1k..64k; one
    token per sequence appended per step into freed slots first"""
    wl = synth.config_stress(n_layers=2, n_steps=64)
    longest, shortest = int(np.argmax(wl.q_pos)), int(np.argmin(wl.q_pos))
    _run(wl, [(longest, 0), (shortest, 1), (128, 1), (7, 0), (200, 0), (255, 1), (64, 0), (31, 1)])
