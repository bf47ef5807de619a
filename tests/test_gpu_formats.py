"""The paper's number formats on the device (THINKV_FMT_FP: E4M3 with a per-tensor scale, E2M1 and ternary codes
with an E4M3 scale per 16 channels) against the oracle (oracle/formats.py through the oracle cache): codes, scale
bytes and every table bit for bit, attention -- the matrix-core kernel and the plain one -- within the tolerance of
the other GPU tests (needs an MI355X)."""
import numpy as np
import pytest
import torch

import parity
from paper_2510_01290_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("bits,scale", [((2, 4, 8), (0.05, 0.07)), ((8, 2, 4), (0.02, 0.5)), ((2, 4, 4), (1.0, 1.0))],
                         ids=["paper-R8E4T2", "T8E2R4", "paper-R4E4T2"])
def test_config1_tiny_in_the_papers_formats(bits, scale):
    _say(f"config 1 tiny in FP8 / NVFP4 / ternary, bits(T,E,R)={bits}, tensor scales {scale} (0.02: values beyond 448 * 0.02 saturate)")
    case = parity.case_tiny(0, bits)
    case.wl.geom.fmt, case.wl.geom.fp8_scale = "fp", scale
    _say(parity.run_case(case, out_dtypes=(torch.float32, torch.float16)))


@pytest.mark.parametrize("D,dtype,G", [(128, "bf16", 4), (64, "f16", 8), (128, "f16", 5), (64, "bf16", 4), (128, "bf16", 1)])
def test_ragged_multi_sequence_with_a_window_layer_in_the_papers_formats(D, dtype, G):
    _say(f"ragged multi-seq in the paper's formats, D={D} {dtype} G={G}, layer 1 with a window of 128")
    geom = synth.Geometry(2, 2 * G, 2, D, dtype, (2, 4, 8), "fp", (0.04, 0.06))
    wl = synth.bulk_evict_refill("ragged-fp", geom, 6, 4, np.array([300, 17, 1000, 1]), {synth.E: 0.3, synth.R: 0.1, synth.T: 0.05},
                                 refill_chunk=3, window_of_layer=[0, 128])
    _say(parity.run_case(parity.Case(wl), out_dtypes=(torch.float32, torch.bfloat16)))


@pytest.mark.parametrize("bulk", [True, False], ids=["bulk-kernel", "per-token-kernel"])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_encoders_on_every_binary16_value(bits, bulk):
    """all finite binary16 values as group members (groups of 16: two fixed members set the scale, fourteen vary) and as
    FP8 inputs: codes and scale bytes from the device equal the oracle's, byte for byte.  Scale-setting members are chosen so
    that ties, saturation (values up to 65504 against a scale of 448 at most) and the subnormal codes all occur."""
    _say(f"exhaustive binary16 encoder check, {bits}-bit type of the paper's formats")
    allv = np.arange(65536, dtype=np.uint16).view(np.float16)
    vals = allv[np.isfinite(allv)]
    rows = []
    for top in (np.float16(6.0), np.float16(0.75), np.float16(40.0), np.float16(3000.0), np.float16(0.0117)):
        sel = vals if top == np.float16(3000.0) else vals[np.abs(vals.astype(np.float32)) <= float(top)]
        n_grp = (len(sel) + 13) // 14
        pad = np.zeros(n_grp * 14, dtype=np.float16)
        pad[:len(sel)] = sel
        r = np.empty((n_grp, 16), dtype=np.float16)
        r[:, 0], r[:, 1], r[:, 2:] = top, -top, pad.reshape(n_grp, 14)
        rows.append(r)
    rows = np.concatenate(rows)
    n_tok = (len(rows) + 7) // 8                   # D=64, Hkv=2: eight groups of 16 per token
    buf = np.zeros((n_tok * 8, 16), dtype=np.float16)
    buf[:len(rows)] = rows
    k = torch.from_numpy(buf.reshape(n_tok, 2, 64))
    v = torch.from_numpy(buf[::-1].copy().reshape(n_tok, 2, 64))
    geom = synth.Geometry(1, 2, 2, 64, "f16", (bits, bits, bits), "fp", (0.37, 3.0))
    wl = synth.Workload("exhaustive-fp", geom, 0, 1, [np.ones(n_tok, np.uint8)], [])
    gc = parity.make_gpu_cache(wl)
    ob = parity.make_oracle(wl)
    ts, tp, tc = np.zeros(n_tok, np.int32), np.arange(n_tok, dtype=np.int32), np.ones(n_tok, np.uint8)
    kd, vd = k.cuda(), v.cuda()
    if not bulk:      # rows that are not 16-byte aligned take the per-token kernel
        kd = torch.cat([kd.flatten()[:1], kd.flatten()])[1:].view(k.shape)
        vd = torch.cat([vd.flatten()[:1], vd.flatten()])[1:].view(v.shape)
        assert kd.data_ptr() % 16 and kd.is_contiguous()
    hg = parity.GpuBackend(gc).append(0, kd, vd, ts, tp, tc)
    ho = ob.append(0, k, v, ts, tp, tc)
    assert np.array_equal(hg, ho)
    parity.compare_bookkeeping_full(ob.cache, gc)
    parity.compare_sequences(ob.cache, gc, [(0, 0, 0)], check_bytes=True)


def test_kmeans_survivors_in_the_papers_formats():
    """thought-adaptive eviction clusters the stored keys, whatever their format"""
    from paper_2510_01290_amd import binding as B
    from oracle import tbe as otbe
    geom = synth.Geometry(1, 8, 2, 64, "f16", (2, 4, 8), "fp", (0.05, 0.05))
    wl = synth.bulk_evict_refill("tbe-fp", geom, 12, 1, np.array([400]), {}, refill=0)
    gc = parity.make_gpu_cache(wl)
    gr = synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    ob = parity.make_oracle(wl)
    synth.ScriptRunner(wl, ob).run()
    hs = gr.handle[(0, 0)]
    cls = wl.classes[0]
    edges = np.r_[0, np.flatnonzero(np.diff(cls)) + 1, len(cls)]
    th, off = [], [0]
    for a, b in zip(edges[:-1], edges[1:]):
        th += [int(h) for h in hs[a:min(b, a + 192)]]
        off.append(len(th))
    th, off = np.array(th, np.int32), np.array(off, np.int32)
    keep = np.full(len(off) - 1, 16, np.int32)
    ts = np.zeros(len(th), np.int32)
    d = gc.device
    ev = torch.empty(len(th), dtype=torch.int32, device=d)
    B.thinkv_tbe_select(gc, 0, torch.from_numpy(ts).to(d), torch.from_numpy(th).to(d), torch.from_numpy(off).to(d), torch.from_numpy(keep).to(d), ev)
    got = ev.cpu().numpy()
    want, margins = otbe.select_evictions(ob.cache, 0, ts, th, off, keep, 8)
    n_clear = 0
    for sg, (a, b) in enumerate(zip(off[:-1], off[1:])):
        if margins[sg] > 3e-5:
            n_clear += 1
            assert np.array_equal(got[a:b], want[a:b]), (sg, margins[sg])
    assert n_clear >= 1
