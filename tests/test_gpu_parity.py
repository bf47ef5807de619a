"""HIP path vs CPU oracle on the same seeded inputs (needs an MI355X)."""
import numpy as np
import pytest
import torch

import backends
import parity
from oracle import cache as ocache
from paper_2510_01290_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("bits", [(8, 2, 4), (2, 4, 8), (2, 4, 4)], ids=["T8E2R4", "paper-R8E4T2", "paper-R4E4T2"])
def test_config1_tiny(bits):
    _say(f"config 1 tiny, bits(T,E,R)={bits}")
    res = parity.run_case(parity.case_tiny(0, bits), out_dtypes=(torch.float32, torch.float16))
    _say(res)


@pytest.mark.parametrize("D,dtype,G", [(128, "bf16", 4), (64, "bf16", 8), (128, "f16", 5), (64, "f16", 1)])
def test_ragged_multi_sequence_multi_layer(D, dtype, G):
    _say(f"ragged multi-seq D={D} {dtype} G={G}")
    geom = synth.Geometry(2, 2 * G, 2, D, dtype, (8, 2, 4))
    wl = synth.bulk_evict_refill("ragged", geom, 5, 4, np.array([300, 17, 1000, 1]), {synth.E: 0.3, synth.R: 0.1, synth.T: 0.05},
                                 refill_chunk=3)
    res = parity.run_case(parity.Case(wl), out_dtypes=(torch.float32, torch.bfloat16))
    _say(res)


def test_budgeted_decode_scrambles_slots():
    _say("config-3-like budgeted decode, scaled down")
    geom = synth.Geometry(1, 10, 2, 128, "bf16", (8, 2, 4))
    wl = synth.budgeted_decode("budget-small", geom, 2, 3, 3000, 512, steps_per_call=8)
    res = parity.run_case(parity.Case(wl))
    _say(res)


def test_sliding_window_layer():
    _say("sliding window W=128 on layer 1")
    geom = synth.Geometry(2, 16, 2, 64, "bf16", (8, 2, 4))
    wl = synth.bulk_evict_refill("window", geom, 9, 3, np.array([700, 90, 2000]), {synth.T: 0.2, synth.E: 0.2, synth.R: 0.2},
                                 refill_chunk=5, window_of_layer=[0, 128])
    res = parity.run_case(parity.Case(wl))
    _say(res)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantizer_every_binary16_value_in_range(bits):
    """all binary16 values in [-8, 8] as group members next to a fixed minimum -8 and maximum 8:
    codes, scales and zero-points from the device equal the oracle's, byte for byte"""
    _say(f"exhaustive binary16 quantizer check, {bits} bits")
    allv = np.arange(65536, dtype=np.uint16).view(np.float16)
    vals = allv[np.isfinite(allv) & (np.abs(allv.astype(np.float32)) <= 8)]
    n_grp = (len(vals) + 29) // 30
    pad = np.zeros(n_grp * 30, dtype=np.float16)
    pad[:len(vals)] = vals
    rows = np.empty((n_grp, 32), dtype=np.float16)
    rows[:, 0], rows[:, 1], rows[:, 2:] = -8, 8, pad.reshape(n_grp, 30)
    n_tok = (n_grp + 3) // 4                       # D=64, Hkv=2: four groups per token
    buf = np.zeros((n_tok * 4, 32), dtype=np.float16)
    buf[:n_grp] = rows
    k = torch.from_numpy(buf.reshape(n_tok, 2, 64))
    v = torch.from_numpy(buf[::-1].copy().reshape(n_tok, 2, 64))
    geom = synth.Geometry(1, 2, 2, 64, "f16", (bits, bits, bits))
    wl = synth.Workload("exhaustive", geom, 0, 1, [np.ones(n_tok, np.uint8)], [])
    gc = parity.make_gpu_cache(wl)
    ob = parity.make_oracle(wl)
    ts, tp, tc = np.zeros(n_tok, np.int32), np.arange(n_tok, dtype=np.int32), np.ones(n_tok, np.uint8)
    hg = parity.GpuBackend(gc).append(0, k.cuda(), v.cuda(), ts, tp, tc)
    ho = ob.append(0, k, v, ts, tp, tc)
    assert np.array_equal(hg, ho)
    parity.compare_bookkeeping_full(ob.cache, gc)
    parity.compare_sequences(ob.cache, gc, [(0, 0, 0)], check_bytes=True)


def test_flags_and_degenerate_cases():
    _say("device-side flags, empty and fully evicted sequences, single token")
    from paper_2510_01290_amd import binding as B
    geom = synth.Geometry(1, 8, 2, 64, "f16", (8, 2, 4))
    wl = synth.Workload("flags", geom, 0, 4, [np.zeros(64, np.uint8)] * 4, [], (0,), np.zeros(4, np.int32))
    gc = parity.make_gpu_cache(wl, arena_pages=(2, 2, 2), max_pages=4)
    ob = parity.make_oracle(wl, arena_pages=(2, 2, 2), max_pages=4)
    gb = parity.GpuBackend(gc)
    dev = gc.device

    def both(seqs, pos, cls, seed):
        n = len(seqs)
        k = synth.normals((seed, 1), 0, n * 2 * 64, "cpu").view(n, 2, 64).to(torch.float16)
        v = synth.normals((seed, 2), 0, n * 2 * 64, "cpu").view(n, 2, 64).to(torch.float16)
        a = gb.append(0, k.to(dev), v.to(dev), np.array(seqs), np.array(pos), np.array(cls, dtype=np.uint8))
        b = ob.append(0, k, v, np.array(seqs), np.array(pos), np.array(cls, dtype=np.uint8))
        assert np.array_equal(a, b), (a, b)
        return a

    h0 = both([0] * 40, list(range(40)), [0] * 40, 1)            # type-0 pool (2 pages) runs dry at 32
    assert (h0[32:] == -1).all()
    h1 = both([1, 1, 1, 2, 9], [0, 1, 2, 0, 0], [1, 7, 2, 2, 1], 2)   # bad class 7, bad sequence 9
    assert h1[1] == -1 and h1[4] == -1
    for seqs, hs in ([[1, 1], [h1[0], h1[0]]], [[1], [ocache.make_handle(2, 3, 0)]], [[2], [h1[3]]], [[7], [0]]):
        gb.evict(0, np.array(seqs), np.array(hs))
        ob.evict(0, np.array(seqs), np.array(hs))
    parity.compare_bookkeeping_full(ob.cache, gc)
    st = gc.dev_status.cpu().numpy()
    assert st[0] & B.ST_NOPAGES and st[1] & B.ST_BAD_CLASS and st[1] & B.ST_EVICT_DEAD and st[1] & B.ST_BAD_SLOT
    assert st[-1] & B.ST_BAD_SEQ
    # sequence 1 keeps a single live token (class R); sequence 2 is fully evicted; sequence 3 never used
    wl.q_pos = np.array([39, 2, 0, 0], dtype=np.int32)
    ref, ref_lse = parity.oracle_attention(ob.cache, wl, 0, [0, 1, 2, 3], [0, 1, 2, 3])
    for variant in ("fast", "valu"):
        got, lse = parity.gpu_attention(gc, wl, None, 0, torch.float32, variant, max_ctx_pages=4)
        assert np.abs(got - ref).max() <= parity.TOL
        assert not got[2].any() and not got[3].any() and np.all(np.isneginf(lse[2:]))
        assert np.abs(got[1] - ref[1]).max() <= 1e-6               # one live token: its value row
        assert np.abs(lse[:2] - ref_lse[:2]).max() <= 1e-3
    # more queries in one call than the view has rows of work counters for: refused, not run
    q5 = torch.zeros((5, 8, 64), dtype=torch.float16, device=dev)
    out5 = torch.zeros((5, 8, 64), dtype=torch.float32, device=dev)
    seq5 = torch.zeros(5, dtype=torch.int32, device=dev)
    with pytest.raises(RuntimeError, match="invalid argument"):
        B.thinkv_decode_attention(gc, 0, q5, out5, None, seq5, None, 0, 0.125, 4)


def test_sequences_compete_for_the_last_pages_in_one_call():
    _say("one append call in which four sequences want more new pages than the pools hold")
    from paper_2510_01290_amd import binding as B
    geom = synth.Geometry(1, 8, 2, 64, "f16", (8, 2, 4))
    wl = synth.Workload("pool", geom, 0, 4, [np.zeros(64, np.uint8)] * 4, [], (0,), np.zeros(4, np.int32))
    # type 0: five pages for 4 x 2 wanted; type 1: three pages for 1 + 2 + 2 wanted; type 2 untouched
    gc = parity.make_gpu_cache(wl, arena_pages=(5, 3, 2), max_pages=4)
    ob = parity.make_oracle(wl, arena_pages=(5, 3, 2), max_pages=4)
    gb = parity.GpuBackend(gc)
    seqs, pos, cls = [], [], []
    for s, (n0, n1) in enumerate([(20, 5), (30, 0), (17, 20), (32, 18)]):   # tokens of type 0 / type 1 per sequence
        c = [0] * n0 + [1] * n1
        rng = np.random.default_rng(100 + s)
        rng.shuffle(c)
        seqs += [s] * len(c)
        pos += list(range(len(c)))
        cls += c
    n = len(seqs)
    k = synth.normals((7, 1), 0, n * 2 * 64, "cpu").view(n, 2, 64).to(torch.float16)
    v = synth.normals((7, 2), 0, n * 2 * 64, "cpu").view(n, 2, 64).to(torch.float16)
    a = gb.append(0, k.to(gc.device), v.to(gc.device), np.array(seqs), np.array(pos), np.array(cls, dtype=np.uint8))
    b = ob.append(0, k, v, np.array(seqs), np.array(pos), np.array(cls, dtype=np.uint8))
    assert np.array_equal(a, b), (a, b)
    assert (a == -1).any() and (a != -1).any()
    parity.compare_bookkeeping_full(ob.cache, gc)
    st = gc.dev_status.cpu().numpy()
    # type 0: sequences 0 and 1 get two pages each, sequence 2 the last one, sequence 3 none
    assert np.array_equal(gc.n_pages[:, 0, 0].cpu().numpy(), [2, 2, 1, 0])
    assert np.array_equal(gc.n_pages[:, 0, 1].cpu().numpy(), [1, 0, 2, 0])
    assert [bool(x & B.ST_NOPAGES) for x in st[:4]] == [False, False, True, True]
    assert gc.free_top.cpu().numpy().tolist() == [0, 0, 2]
    # a second call finds the pools empty for types 0 and 1 and still fills the tails that are left
    seqs2, pos2, cls2 = [0] * 14, list(range(100, 114)), [0] * 14                  # sequence 0: 12 free slots in its last page
    k2 = synth.normals((8, 1), 0, 14 * 2 * 64, "cpu").view(14, 2, 64).to(torch.float16)
    a2 = gb.append(0, k2.to(gc.device), k2.to(gc.device), np.array(seqs2), np.array(pos2), np.array(cls2, dtype=np.uint8))
    b2 = ob.append(0, k2, k2, np.array(seqs2), np.array(pos2), np.array(cls2, dtype=np.uint8))
    assert np.array_equal(a2, b2) and (a2[:12] != -1).all() and (a2[12:] == -1).all()
    parity.compare_bookkeeping_full(ob.cache, gc)
    parity.compare_sequences(ob.cache, gc, [(s, s, 0) for s in range(4)], check_bytes=True)


def test_window_with_positions_out_of_order():
    _say("sliding window over pages whose positions were written out of order and reused")
    geom = synth.Geometry(1, 8, 2, 64, "f16", (8, 2, 4))
    n = 96
    wl = synth.Workload("winpos", geom, 3, 1, [np.zeros(4096, np.uint8)], [], (40,), np.array([2000], np.int32))
    gc = parity.make_gpu_cache(wl, arena_pages=(8, 8, 8), max_pages=8)
    ob = parity.make_oracle(wl, arena_pages=(8, 8, 8), max_pages=8)
    gb = parity.GpuBackend(gc)
    rng = np.random.default_rng(5)
    # 96 tokens over three types with positions in a scrambled order: recent and old positions share pages
    pos = rng.permutation(np.arange(1900, 1900 + n)).astype(np.int64)
    cls = rng.integers(0, 3, size=n).astype(np.uint8)
    k = synth.normals((9, 1), 0, n * 2 * 64, "cpu").view(n, 2, 64).to(torch.float16)
    v = synth.normals((9, 2), 0, n * 2 * 64, "cpu").view(n, 2, 64).to(torch.float16)
    ha = gb.append(0, k.to(gc.device), v.to(gc.device), np.zeros(n, np.int64), pos, cls)
    hb = ob.append(0, k, v, np.zeros(n, np.int64), pos, cls)
    assert np.array_equal(ha, hb)
    # evict the most recent third (their positions stay behind as the pages' upper bounds), refill with old positions
    ev = ha[np.argsort(pos)[-32:]]
    gb.evict(0, np.zeros(32, np.int64), ev)
    ob.evict(0, np.zeros(32, np.int64), ev)
    pos2 = np.arange(100, 116, dtype=np.int64)
    cls2 = rng.integers(0, 3, size=16).astype(np.uint8)
    k2 = synth.normals((9, 3), 0, 16 * 2 * 64, "cpu").view(16, 2, 64).to(torch.float16)
    assert np.array_equal(gb.append(0, k2.to(gc.device), k2.to(gc.device), np.zeros(16, np.int64), pos2, cls2),
                          ob.append(0, k2, k2, np.zeros(16, np.int64), pos2, cls2))
    parity.compare_bookkeeping_full(ob.cache, gc)
    for qp in (1995, 1940, 1966, 130, 50):
        wl.q_pos = np.array([qp], dtype=np.int32)
        ref, ref_lse = parity.oracle_attention(ob.cache, wl, 0, [0], [0])
        for variant in ("fast", "valu"):
            got, lse = parity.gpu_attention(gc, wl, None, 0, torch.float32, variant, max_ctx_pages=24)
            assert np.abs(got - ref).max() <= parity.TOL, (qp, variant, np.abs(got - ref).max())
            fin = np.isfinite(ref_lse)
            assert np.array_equal(np.isfinite(lse), fin)
            assert not fin.any() or np.abs(lse[fin] - ref_lse[fin]).max() <= 1e-3
            assert fin.any() or not got.any()                      # nothing visible: zeros and -inf


def test_decode_calls_replay_correctly_from_a_captured_graph():
    _say("decode attention (plain and with the sparsity statistic) captured in a graph, replayed between eager calls")
    from paper_2510_01290_amd import binding as B
    geom = synth.Geometry(1, 8, 2, 128, "bf16", (8, 2, 4))
    wl = synth.bulk_evict_refill("graph", geom, 13, 3, np.array([900, 40, 2500]), {synth.E: 0.3}, refill_chunk=4)
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    dev = gc.device
    seqs = list(range(wl.n_seqs))
    q = torch.stack([synth.query_rows(wl.seed, 0, s, 0, geom, dev) for s in seqs]).contiguous()
    sid = torch.tensor(seqs, dtype=torch.int32, device=dev)
    qp = torch.from_numpy(wl.q_pos.astype(np.int32)).to(dev)
    mcp = int(gc.n_pages[:, 0].sum(-1).max().item())
    scale = geom.head_dim ** -0.5
    outs = [torch.empty(q.shape, dtype=torch.float32, device=dev) for _ in range(3)]
    lses = [torch.empty((len(seqs), geom.n_q_heads), dtype=torch.float32, device=dev) for _ in range(3)]
    sps = [torch.empty(len(seqs), dtype=torch.float32, device=dev) for _ in range(2)]
    # eager reference (also sizes the workspace, so nothing is allocated while capturing)
    B.thinkv_decode_attention_sparsity(gc, 0, q, outs[0], lses[0], sps[0], sid, qp, 0, scale, mcp)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.thinkv_decode_attention(gc, 0, q, outs[1], lses[1], sid, qp, 0, scale, mcp)
            B.thinkv_decode_attention_sparsity(gc, 0, q, outs[2], lses[2], sps[1], sid, qp, 0, scale, mcp)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs[1:] + lses[1:] + sps[1:]:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for o in outs[1:]:
            assert float((o - outs[0]).abs().max()) <= 1e-4, rep          # the split of the work differs from run to run
        assert torch.equal(sps[1], sps[0]), rep
        assert int(gc.work_counters.abs().sum().item()) == 0, "work counters not back at zero"
        # eager work between the replays
        B.thinkv_decode_attention(gc, 0, q, outs[0].clone(), None, sid, qp, 0, scale, mcp)
        torch.cuda.synchronize()


@pytest.mark.parametrize("D,dtype,shift", [(128, torch.float32, 0), (64, torch.float32, 0), (128, torch.bfloat16, 1),
                                           (64, torch.float16, 3), (128, torch.float32, 1)])
def test_bulk_append_input_formats(D, dtype, shift):
    _say(f"bulk append: D={D} {dtype}, rows start {shift} elements off a 16-byte boundary, types mixed token by token, "
         "evictions between two calls")
    H, n_tok = 3, 700
    geom = synth.Geometry(1, 2 * H, H, D, "f16", (8, 2, 4))
    rng = np.random.default_rng(77 + D + shift)
    cls = rng.integers(0, 3, n_tok).astype(np.uint8)
    wl = synth.Workload("bulk-formats", geom, 0, 2, [np.concatenate([cls, cls]), np.concatenate([cls, cls])], [])
    gc = parity.make_gpu_cache(wl)
    ob = parity.make_oracle(wl)
    gb = parity.GpuBackend(gc)

    def rows(seed):
        g = torch.Generator().manual_seed(seed)
        flat = (torch.randn(2 * n_tok * H * D + 8, generator=g) * 3).to(dtype)
        return flat[shift:shift + 2 * n_tok * H * D].view(2 * n_tok, H, D)      # a view: not contiguous-copied below

    ts = np.repeat(np.arange(2, dtype=np.int32), n_tok)
    tp = np.tile(np.arange(n_tok, dtype=np.int32), 2)
    tc = np.tile(cls, 2)
    for call in range(2):
        k, v = rows(10 + call), rows(20 + call)
        kd, vd = k.cuda(), v.cuda()
        if shift:   # .cuda() of a view keeps no offset: rebuild the offset on the device
            fk = torch.empty(kd.numel() + 8, dtype=dtype, device="cuda")
            fv = torch.empty(kd.numel() + 8, dtype=dtype, device="cuda")
            fk[shift:shift + kd.numel()] = kd.reshape(-1)
            fv[shift:shift + vd.numel()] = vd.reshape(-1)
            kd, vd = fk[shift:shift + kd.numel()].view(k.shape), fv[shift:shift + vd.numel()].view(v.shape)
            assert kd.data_ptr() % 16 != 0
        from paper_2510_01290_amd import binding as B
        d = gc.device
        h = torch.empty(len(ts), dtype=torch.int32, device=d)
        B.thinkv_append_quantized(gc, 0, kd, vd, torch.from_numpy(ts).to(d), torch.from_numpy(tp + call * n_tok).to(d),
                                  torch.from_numpy(tc).to(d), h)
        hg = h.cpu().numpy()
        ho = ob.append(0, k, v, ts, tp + call * n_tok, tc)
        assert np.array_equal(hg, ho), call
        if call == 0:   # free a third of the slots: the second call reuses them in place before it takes new pages
            pick = rng.random(len(hg)) < 0.33
            gb.evict(0, ts[pick], hg[pick])
            ob.evict(0, ts[pick], ho[pick])
    assert int(gc.dev_status.abs().sum().item()) == 0
    parity.compare_bookkeeping_full(ob.cache, gc)
    parity.compare_sequences(ob.cache, gc, [(0, 0, 0), (1, 1, 0)], check_bytes=True)


@pytest.mark.parametrize("seed,D,fused", [(1, 64, False), (2, 128, False), (3, 64, True), (4, 128, True), (5, 128, True)])
def test_random_operation_sequences(seed, D, fused):
    _say(f"random appends (1 .. 300 tokens a call, both append paths) and evictions (live, dead, repeated, placeholder handles) "
         f"on small pools and short page lists, seed {seed}, D={D}" + (", evictions handed over with the next append (thinkv_evict_append)" if fused else ""))
    from paper_2510_01290_amd import binding as B
    H, S = 2, 5
    geom = synth.Geometry(1, 2 * H, H, D, "f16", (8, 2, 4) if seed % 2 else (2, 4, 8))
    wl = synth.Workload("fuzz", geom, seed, S, [np.zeros(16, np.uint8)] * S, [], (0,), np.zeros(S, np.int32))
    arena, max_pages = (14, 10, 12), 6                       # both the pools and the page lists run out now and then
    gc = parity.make_gpu_cache(wl, arena_pages=arena, max_pages=max_pages)
    ob = parity.make_oracle(wl, arena_pages=arena, max_pages=max_pages)
    gb = parity.GpuBackend(gc)
    rng = np.random.default_rng(1000 + seed)
    next_pos = np.zeros(S, np.int64)
    live = [dict() for _ in range(S)]                        # handle -> True, per sequence, as the calls returned them
    dead = [[] for _ in range(S)]
    n_calls = {"small": 0, "bulk": 0, "evict": 0, "fused": 0, "tokens_without_a_slot": 0}
    pending = None
    for op in range(36):
        if op % 3 != 2 or not any(live):
            seqs, cls = [], []
            for s in sorted(rng.choice(S, size=int(rng.integers(1, S + 1)), replace=False).tolist()):
                n = int(rng.choice([1, 1, 1, 2, 5, 17, 40, 120]))
                seqs += [s] * n
                bias = rng.dirichlet([1.0, 1.0, 1.0])
                cls += rng.choice(3, size=n, p=bias).tolist()
            n = len(seqs)
            seqs, cls = np.array(seqs, np.int32), np.array(cls, np.uint8)
            pos = np.empty(n, np.int32)
            for s in range(S):
                m = seqs == s
                pos[m] = next_pos[s] + np.arange(int(m.sum()))
                next_pos[s] += int(m.sum())
            g = torch.Generator().manual_seed(seed * 1000 + op)
            k = (torch.randn((n, H, D), generator=g) * float(rng.uniform(0.1, 8))).to(torch.float16)
            v = (torch.randn((n, H, D), generator=g) * float(rng.uniform(0.1, 8))).to(torch.float16)
            if pending is not None:
                d = gc.device
                h = torch.empty(n, dtype=torch.int32, device=d)
                B.thinkv_evict_append(gc, 0, torch.from_numpy(pending[0]).to(d), torch.from_numpy(pending[1]).to(d),
                                      k.to(d), v.to(d), torch.from_numpy(seqs).to(d), torch.from_numpy(pos).to(d),
                                      torch.from_numpy(cls).to(d), h)
                hg = h.cpu().numpy()
                pending = None
                n_calls["fused"] += 1
            else:
                hg = gb.append(0, k.to(gc.device), v.to(gc.device), seqs, pos, cls)
            ho = ob.append(0, k, v, seqs, pos, cls)
            assert np.array_equal(hg, ho), ("handles", op, n)
            n_calls["small" if n <= 64 else "bulk"] += 1
            n_calls["tokens_without_a_slot"] += int((hg == -1).sum())
            for s, h in zip(seqs.tolist(), hg.tolist()):
                if h != -1:
                    live[s][h] = True
        else:
            es, eh = [], []
            for s in range(S):
                hs = np.array(list(live[s].keys()), dtype=np.int64)
                if hs.size:
                    pick = hs[rng.random(hs.size) < rng.choice([0.1, 0.5, 0.9])]
                    es += [s] * pick.size
                    eh += pick.tolist()
                    for h in pick.tolist():
                        del live[s][h]
                        dead[s].append(h)
                if dead[s] and rng.random() < 0.3:             # a slot that is already dead, and a placeholder
                    es += [s, s]
                    eh += [int(rng.choice(dead[s])), -1]
            if eh and rng.random() < 0.5:                      # the same live handle twice in one call counts once
                es.append(es[0])
                eh.append(eh[0])
            if rng.random() < 0.3:                             # a sequence that does not exist
                es.append(S + 3)
                eh.append(0)
            order = rng.permutation(len(eh))
            es, eh = np.array(es, np.int32)[order], np.array(eh, np.int32)[order]
            if fused and len(eh):
                pending = (es, eh)          # the device gets them with the next append
            else:
                gb.evict(0, es, eh)
            ob.evict(0, es, eh)
            n_calls["evict"] += 1
            # (a "dead" handle whose slot was refilled meanwhile kills a live token, on both sides alike;
            # the lists above only steer the choice of handles)
        if op % 6 == 5 and pending is None:
            parity.compare_bookkeeping_full(ob.cache, gc)
    if pending is not None:
        gb.evict(0, *pending)
    parity.compare_bookkeeping_full(ob.cache, gc)
    parity.compare_sequences(ob.cache, gc, [(s, s, 0) for s in range(S)], check_bytes=True)
    assert n_calls["small"] and n_calls["bulk"] and n_calls["evict"] and n_calls["tokens_without_a_slot"], n_calls
    assert bool(n_calls["fused"]) == fused
    # attention over what is left, both kernels
    wl.q_pos = next_pos.astype(np.int32)
    ref, ref_lse = parity.oracle_attention(ob.cache, wl, 0, list(range(S)), list(range(S)))
    for variant in ("fast", "valu"):
        got, lse = parity.gpu_attention(gc, wl, None, 0, torch.float32, variant)
        assert float(np.abs(got - ref).max()) <= parity.TOL, variant
    _say(n_calls)


def test_whole_decode_step_replays_correctly_from_a_captured_graph():
    _say("evict + append (one call) + decode attention captured in a graph on one cache, replayed three times; "
         "the same steps run eagerly on a twin cache")
    from paper_2510_01290_amd import binding as B
    geom = synth.Geometry(1, 8, 2, 128, "bf16", (8, 2, 4))
    wl = synth.bulk_evict_refill("graph-step", geom, 17, 3, np.array([700, 90, 1500]), {synth.E: 0.2}, refill_chunk=4)
    twins = []
    for _ in range(2):
        gc = parity.make_gpu_cache(wl)
        gr = synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
        twins.append(gc)
    eager, graphed = twins
    dev, S = eager.device, wl.n_seqs
    # static inputs of the captured step; their contents change between replays
    hs = [gr.handle[(0, s)] for s in range(S)]
    live = [[int(h) for h in hs[s][:60] if h != -1] for s in range(S)]
    ev_seq = torch.arange(S, dtype=torch.int32, device=dev)
    ev_h = torch.zeros(S, dtype=torch.int32, device=dev)
    k = torch.zeros((S, geom.n_kv_heads, geom.head_dim), dtype=torch.bfloat16, device=dev)
    v = torch.zeros_like(k)
    pos = torch.zeros(S, dtype=torch.int32, device=dev)
    cls = torch.zeros(S, dtype=torch.uint8, device=dev)
    q = torch.zeros((S, geom.n_q_heads, geom.head_dim), dtype=torch.bfloat16, device=dev)
    mcp = int(eager.n_pages[:, 0].sum(-1).max().item()) + 2
    scale = geom.head_dim ** -0.5
    outs = {c: torch.empty(q.shape, dtype=torch.float32, device=dev) for c in ("eager", "graph")}
    hnd = {c: torch.empty(S, dtype=torch.int32, device=dev) for c in ("eager", "graph")}

    def step(gc, tag):
        B.thinkv_evict_append(gc, 0, ev_seq, ev_h, k, v, ev_seq, pos, cls, hnd[tag])
        B.thinkv_decode_attention(gc, 0, q, outs[tag], None, ev_seq, pos, 0, scale, mcp)

    def set_inputs(i):
        ev_h.copy_(torch.tensor([live[s][i] for s in range(S)], dtype=torch.int32))
        k.copy_(torch.stack([synth.kv_rows(wl.seed, 0, s, 0, 5000 + i, 5001 + i, geom, dev)[0] for s in range(S)]))
        v.copy_(torch.stack([synth.kv_rows(wl.seed, 0, s, 1, 5000 + i, 5001 + i, geom, dev)[0] for s in range(S)]))
        pos.copy_(torch.tensor([int(wl.q_pos[s]) + 1 + i for s in range(S)], dtype=torch.int32))
        cls.copy_(torch.tensor([(s + i) % 3 for s in range(S)], dtype=torch.uint8))
        q.copy_(torch.stack([synth.query_rows(wl.seed, 0, s, 100 + i, geom, dev) for s in range(S)]))

    set_inputs(0)
    step(eager, "eager")                       # also sizes the workspaces, so nothing is allocated while capturing
    graphed.workspace(max(int(eager._ws.numel()) if getattr(eager, "_ws", None) is not None else 0, 1 << 20))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.thinkv_decode_attention(graphed, 0, q, outs["graph"], None, ev_seq, pos, 0, scale, mcp)   # warm-up on the side stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(graphed, "graph")
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for i in range(3):
        if i:
            set_inputs(i)
            step(eager, "eager")
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(hnd["eager"], hnd["graph"]), i
        assert float((outs["eager"] - outs["graph"]).abs().max()) <= 1e-4, i
        for name in ("block_table", "slot_mask", "n_pages", "n_live", "dev_status", "free_top", "work_counters", "append_counters"):
            assert torch.equal(getattr(eager, name), getattr(graphed, name)), (name, i)
        for c in range(3):
            assert torch.equal(eager.arena[c], graphed.arena[c]), ("arena", c, i)
            assert torch.equal(eager.slot_pos[c], graphed.slot_pos[c]), ("slot_pos", c, i)
    assert int(eager.dev_status.abs().sum().item()) == 0


def test_context_bound_below_the_true_page_count_still_attends_everything():
    """max_ctx_pages is the host's bound for sizing the launch; a sequence that holds more pages than the bound gets fewer
    items than it would like, but every page is still attended (both kernels, full-attention and window layers)"""
    _say("decode attention with a context bound that is too small")
    from paper_2510_01290_amd import binding as B
    geom = synth.Geometry(2, 8, 2, 64, "f16", (8, 2, 4))
    wl = synth.bulk_evict_refill("short-bound", geom, 13, 3, np.array([2500, 40, 900]), {synth.E: 0.2}, refill_chunk=9, window_of_layer=[0, 128])
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    ob = parity.make_oracle(wl)
    synth.ScriptRunner(wl, ob).run()
    for layer in (0, 1):
        ref, ref_lse = parity.oracle_attention(ob.cache, wl, layer, [0, 1, 2], [0, 1, 2])
        true_pages = int(gc.n_pages[:, layer].sum(-1).max().item())
        for bound in (true_pages // 3, 5, 1, 0):
            for variant in ("fast", "valu"):
                out, lse = parity.gpu_attention(gc, wl, None, layer, torch.float32, variant, max_ctx_pages=bound)
                assert np.abs(out - ref).max() <= parity.TOL, (layer, bound, variant, float(np.abs(out - ref).max()))
                assert np.abs(lse - ref_lse).max() <= 1e-3


def test_measurement_aids_run_and_refuse_bad_arguments():
    """thinkv_probe_stream_pages only reads; it must run on any cache (empty sequences, unknown ids) and leave the cache as it was"""
    import ctypes as C
    from paper_2510_01290_amd import binding as B
    geom = synth.Geometry(2, 8, 2, 128, "bf16", (8, 2, 4))
    wl = synth.bulk_evict_refill("probe", geom, 3, 3, np.array([700, 0, 33]), {synth.E: 0.5}, refill_chunk=5)
    wl.classes[1] = np.zeros(0, np.uint8)
    gc = parity.make_gpu_cache(wl)
    synth.ScriptRunner(wl, parity.GpuBackend(gc)).run()
    before = [a.clone() for a in gc.arena] + [gc.block_table.clone(), gc.slot_mask.clone(), gc.work_counters.clone()]
    chk = torch.zeros(1, dtype=torch.int32, device=gc.device)
    for layer in (0, 1):
        B.thinkv_probe_stream_pages(gc, layer, torch.tensor([0, 1, 2, 7, -1], dtype=torch.int32, device=gc.device)[:3], chk)
    torch.cuda.synchronize()
    after = [a for a in gc.arena] + [gc.block_table, gc.slot_mask, gc.work_counters]
    assert all(torch.equal(x, y) for x, y in zip(before, after))
    lib = B.load()
    assert lib.thinkv_probe_stream_pages(C.byref(gc.view), 5, C.c_void_p(chk.data_ptr()), 1, C.c_void_p(chk.data_ptr()), None) == 1
    assert lib.thinkv_probe_stream_pages(C.byref(gc.view), 0, None, 1, C.c_void_p(chk.data_ptr()), None) == 1
    assert lib.thinkv_probe_stream_pages(C.byref(gc.view), 0, None, 0, None, None) == 0
