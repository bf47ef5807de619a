#!/usr/bin/env python3
"""Benchmark of the ThinKV decode hot path on one MI355X.

A step = one pass of the whole path over one batch: soft-evict one token per sequence,
quantise-and-append one new token per sequence (reusing freed slots), decode attention for
every sequence.  Workload: DeepSeek-R1-Distill-Llama-8B-shaped layer (32 query / 8 KV heads,
head_dim 128, bf16), batch 16, 32,768 live tokens per sequence in 16-token pages at
T8/R4/E2 bits, built by bulk append, class-wise eviction (30 % of E, 10 % of R) and refill.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12
# HBM bytes of one decode-attention launch (split-K kernel + merge) on the default workload, from
# rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a copy of known size
# (profiles/decode_attention_cfg2_32k_hbm_traffic.txt); other workloads report null
TRAFFIC_DEFAULT_BYTES = 753.7e6
TRAFFIC_SOURCE = "profiles/decode_attention_cfg2_32k_hbm_traffic.txt (rocprofv3 counters of an earlier run of this command, not measured live)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--ctx", type=int, default=32768, help="live tokens per sequence")
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--variant", default="fast", choices=["fast", "valu"])
    ap.add_argument("--bits", default="8,2,4", help="bit widths of the thought types T,E,R of the default workload (BASELINE: 8,2,4); "
                                                     "8,8,8 / 4,4,4 / 2,2,2 give caches of the same shape with a single width")
    ap.add_argument("--workload", default="cfg2-32k", choices=["cfg2-32k", "cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="cfg2-32k (default): the headline step.  The others time decode attention alone on that "
                         "configuration's cache (a step = one attention call per built layer)")
    ap.add_argument("--format", default="int", choices=["int", "fp"],
                    help="number formats of the default workload's cache: int = integer codes with binary16 scale and zero-point per 32 "
                         "(BASELINE.json); fp = the paper's FP8-E4M3 / NVFP4 / ternary with E4M3 scales per 16")
    ap.add_argument("--replicas", type=int, default=3,
                    help="identical copies of the cache the steps rotate over, so that the data of a step was last touched "
                         "replicas steps ago (3 x 0.75 GB is far beyond the 256 MB memory-side cache)")
    ap.add_argument("--contrast", action="store_true",
                    help="also time what in-place slot reuse avoids: compaction of a contiguous binary16 cache by a gather kernel "
                         "(thinkv_gather_rows) after an eviction, alone and running beside decode attention on a second stream")
    ap.add_argument("--e2e", action="store_true",
                    help="with --workload cfg5: the configuration as written -- 64 consecutive decode steps of {append one token "
                         "per sequence on every layer, an eviction pass every 16th step, attention on every layer}")
    ap.add_argument("--layers", type=int, default=32, help="layers built for --workload cfg5 --e2e (32 = the configuration; fewer is stated in the output)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (gives FETCH_SIZE / WRITE_SIZE a known size to be scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (one MI355X per box); --gpus must be 1")

    import numpy as np
    import torch
    from paper_2510_01290_amd import binding as B
    from paper_2510_01290_amd import synth
    from paper_2510_01290_amd import harness

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "cfg5" and args.e2e:
        print(json.dumps(e2e_cfg5(args, np, torch, B, synth, harness, dev)))
        return
    if args.workload != "cfg2-32k":
        print(json.dumps(attention_only(args, np, torch, B, synth, harness, dev)))
        return
    n_extra = 20   # steps after the timed region, with every call bracketed by events
    nsteps = args.steps + args.warmup + 2 * n_extra
    wl = synth.config_llama8b_layer(seed=1, n_seqs=args.batch, ctx=args.ctx, refill_chunk=64,
                                    name=f"cfg2-shape B={args.batch} ctx={args.ctx}")
    bits = tuple(int(x) for x in args.bits.split(","))
    assert len(bits) == 3 and all(b_ in (2, 4, 8) for b_ in bits)
    wl.geom.bits_of_class = bits
    wl.geom.fmt = args.format
    g = wl.geom
    tok_bytes = [2 * (g.head_dim * b_ // 8 + (g.head_dim // 32 * 4 if args.format == "int" else (0 if b_ == 8 else g.head_dim // 16))) for b_ in bits]
    # room for the timed appends
    arena = tuple(int(x + args.batch * (nsteps // 16 + 2)) for x in harness.arena_need(wl))
    maxp = harness.max_pages_need(wl) + nsteps // 16 + 2
    t0 = time.time()
    gcs = []
    for _ in range(max(1, args.replicas)):
        gc_r = harness.make_gpu_cache(wl, arena_pages=arena, max_pages=maxp)
        gr = synth.ScriptRunner(wl, harness.GpuBackend(gc_r)).run()       # the same script: same handles in every copy
        gcs.append(gc_r)
    gc = gcs[0]
    torch.cuda.synchronize()
    build_s = time.time() - t0
    for gc_r in gcs:
        assert int(gc_r.dev_status.abs().sum().item()) == 0, "device flags set while building the cache"

    # ---- per-step inputs, resident on the device before timing starts
    rng = np.random.default_rng(1234)
    ev_handles = np.empty((nsteps, args.batch), dtype=np.int32)
    new_cls = np.empty((nsteps, args.batch), dtype=np.uint8)
    ntok0 = [len(c) for c in wl.classes]
    for s in range(args.batch):
        hs = gr.handle[(0, s)]
        cls = wl.classes[s]
        # positions still live: never evicted by the build script
        dead = np.zeros(len(hs), dtype=bool)
        for op in wl.ops:
            if isinstance(op, synth.Evict):
                dead[op.pos[op.seqs == s]] = True
        cand = np.flatnonzero((~dead) & (cls == synth.E))
        ev_handles[:, s] = hs[rng.choice(cand, size=nsteps, replace=False)]
        new_cls[:, s] = synth.thought_classes(rng, nsteps)[0]
    ev_seq = torch.arange(args.batch, dtype=torch.int32, device=dev)
    ev_h = torch.from_numpy(ev_handles).to(dev)
    t_cls = torch.from_numpy(new_cls).to(dev)
    t_pos = torch.stack([torch.arange(ntok0[s], ntok0[s] + nsteps, dtype=torch.int32) for s in range(args.batch)], 1).contiguous().to(dev)
    k_new = torch.stack([synth.kv_rows(wl.seed, 0, s, 0, ntok0[s], ntok0[s] + nsteps, g, dev) for s in range(args.batch)], 1).contiguous()
    v_new = torch.stack([synth.kv_rows(wl.seed, 0, s, 1, ntok0[s], ntok0[s] + nsteps, g, dev) for s in range(args.batch)], 1).contiguous()
    # (generated on the host and moved once: a few thousand tiny device launches less)
    cpu = torch.device("cpu")
    q_all = torch.stack([torch.stack([synth.query_rows(wl.seed, 0, s, st, g, cpu) for s in range(args.batch)]) for st in range(nsteps)]).contiguous().to(dev)
    out = torch.empty((args.batch, g.n_q_heads, g.head_dim), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((args.batch, g.n_q_heads), dtype=torch.float32, device=dev)
    h_out = torch.empty(args.batch, dtype=torch.int32, device=dev)
    max_ctx_pages = int(gc.n_pages[:, 0].sum(-1).max().item()) + nsteps // 16 + 3
    scale = g.head_dim ** -0.5
    decode = B.thinkv_decode_attention if args.variant == "fast" else B.thinkv_decode_attention_valu

    def step(i, ev=None):
        gc = gcs[i % len(gcs)]
        B.thinkv_evict_append(gc, 0, ev_seq, ev_h[i], k_new[i], v_new[i], ev_seq, t_pos[i], t_cls[i], h_out)
        if ev is not None:
            ev[0].record()
        decode(gc, 0, q_all[i], out, lse, ev_seq, t_pos[i], 0, scale, max_ctx_pages)
        if ev is not None:
            ev[1].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i, evs[i])
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = e0.elapsed_time(e1) / args.steps
    attn_ms = np.array([a.elapsed_time(b) for a, b in evs])
    # per-call times of the other two entry points, outside the timed region
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_extra)]
    for j in range(n_extra):
        i = args.warmup + args.steps + j
        gc = gcs[i % len(gcs)]
        marks[j][0].record()
        B.thinkv_evict(gc, 0, ev_seq, ev_h[i])
        marks[j][1].record()
        B.thinkv_append_quantized(gc, 0, k_new[i], v_new[i], ev_seq, t_pos[i], t_cls[i], h_out)
        marks[j][2].record()
        decode(gc, 0, q_all[i], out, lse, ev_seq, t_pos[i], 0, scale, max_ctx_pages)
    # the step's two bookkeeping calls as one (what the timed steps use)
    fmarks = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_extra)]
    for j in range(n_extra):
        i = args.warmup + args.steps + n_extra + j
        gc = gcs[i % len(gcs)]
        fmarks[j][0].record()
        B.thinkv_evict_append(gc, 0, ev_seq, ev_h[i], k_new[i], v_new[i], ev_seq, t_pos[i], t_cls[i], h_out)
        fmarks[j][1].record()
        decode(gc, 0, q_all[i], out, lse, ev_seq, t_pos[i], 0, scale, max_ctx_pages)
    gc = gcs[0]
    # decode attention with the attention-sparsity statistic riding on it
    sp = torch.empty(args.batch, dtype=torch.float32, device=dev)
    smarks = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_extra)]
    if args.variant == "fast" and args.format == "int":
        i = nsteps - 1
        for j in range(n_extra + 3):
            gc = gcs[j % len(gcs)]
            if j >= 3:
                smarks[j - 3][0].record()
            B.thinkv_decode_attention_sparsity(gc, 0, q_all[i], out, lse, sp, ev_seq, t_pos[i], 0, scale, max_ctx_pages)
            if j >= 3:
                smarks[j - 3][1].record()
    # bulk (prefill-style) append: 2,048 tokens for each of 16 sequences in one call, type R, into an empty cache
    S_b, n_b = 16, 2048
    bc = B.Cache(1, g.n_q_heads, g.n_kv_heads, g.head_dim, g.bits_of_class, S_b, n_b // 16 + 2, (1, 1, S_b * (n_b // 16) + 8), device=dev)
    kb = torch.randn((S_b * n_b, g.n_kv_heads, g.head_dim), device=dev, dtype=torch.float32).to(k_new.dtype)
    sb = torch.arange(S_b, dtype=torch.int32, device=dev).repeat_interleave(n_b)
    pb = torch.arange(n_b, dtype=torch.int32, device=dev).repeat(S_b)
    cb = torch.full((S_b * n_b,), synth.R, dtype=torch.uint8, device=dev)
    bulk_us = []
    for j in range(4):
        B.thinkv_init_view(bc)
        a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a_.record()
        B.thinkv_append_quantized(bc, 0, kb, kb, sb, pb, cb)
        b_.record()
        torch.cuda.synchronize()
        if j:
            bulk_us.append(a_.elapsed_time(b_) * 1e3)
    assert int(bc.dev_status.abs().sum().item()) == 0 and int(bc.n_live.sum().item()) == S_b * n_b
    bulk = {"tokens": S_b * n_b, "us_median": float(np.median(bulk_us)), "tokens_per_s": S_b * n_b / (float(np.median(bulk_us)) * 1e-6),
            "input_GB_per_s": 2 * kb.numel() * kb.element_size() / (float(np.median(bulk_us)) * 1e-6) / 1e9}
    del bc, kb
    gc = gcs[0]
    # survivor choice of thought-adaptive eviction: 8 segments of 128 consecutive live tokens per sequence, cut to 64
    tbe = None
    if args.variant == "fast":
        t_seq, t_h, off = [], [], [0]
        for s in range(args.batch):
            hs = gr.handle[(0, s)]
            alive = np.flatnonzero(hs[:4096] != -1)
            dead = np.zeros(len(hs), dtype=bool)
            for op in wl.ops:
                if isinstance(op, synth.Evict):
                    dead[op.pos[op.seqs == s]] = True
            alive = alive[~dead[alive]][:1024]
            for a0 in range(0, len(alive) - 127, 128):
                t_seq += [s] * 128
                t_h += [int(x) for x in hs[alive[a0:a0 + 128]]]
                off.append(len(t_h))
        d_seq = torch.tensor(t_seq, dtype=torch.int32, device=dev)
        d_h = torch.tensor(t_h, dtype=torch.int32, device=dev)
        d_off = torch.tensor(off, dtype=torch.int32, device=dev)
        d_keep = torch.full((len(off) - 1,), 64, dtype=torch.int32, device=dev)
        d_ev = torch.empty_like(d_h)
        tm = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        B.thinkv_tbe_select(gc, 0, d_seq, d_h, d_off, d_keep, d_ev)
        for a_, b_ in tm:
            a_.record()
            B.thinkv_tbe_select(gc, 0, d_seq, d_h, d_off, d_keep, d_ev)
            b_.record()
        torch.cuda.synchronize()
        tbe = {"segments": len(off) - 1, "tokens_per_segment": 128, "keep": 64, "max_iters": 8,
               "us_median": float(np.median([a_.elapsed_time(b_) for a_, b_ in tm]) * 1e3),
               "survivors": int((d_ev == -1).sum().item())}
    # the eviction plan on the device: every sequence's segment table (runs of one thought type, at most 192 tokens),
    # a transition has just ended everywhere, so every closed segment above the floor is listed with its live tokens
    plan = None
    if args.variant == "fast":
        max_segs = 2048
        seg_start = np.zeros((args.batch, max_segs), np.int32)
        seg_type = np.zeros((args.batch, max_segs), np.uint8)
        n_segs = np.zeros(args.batch, np.int32)
        for s in range(args.batch):
            cls = wl.classes[s][:ntok0[s]]
            edges = np.r_[0, np.flatnonzero(np.diff(cls)) + 1, len(cls)]
            starts = np.concatenate([np.arange(a0, b0, 192) for a0, b0 in zip(edges[:-1], edges[1:])])[:max_segs]
            n_segs[s] = len(starts)
            seg_start[s, :len(starts)] = starts
            seg_type[s, :len(starts)] = cls[starts]
        cap_seg, cap_tok = args.batch * 256, args.batch * 256 * 192
        p_out = [torch.empty(cap_tok, dtype=torch.int32, device=dev), torch.empty(cap_tok, dtype=torch.int32, device=dev),
                 torch.empty(cap_seg + 1, dtype=torch.int32, device=dev), torch.empty(cap_seg, dtype=torch.int32, device=dev),
                 torch.empty(2, dtype=torch.int32, device=dev)]
        p_in = [ev_seq, torch.from_numpy(seg_start).to(dev), torch.from_numpy(seg_type).to(dev), torch.from_numpy(n_segs).to(dev),
                torch.ones(args.batch, dtype=torch.uint8, device=dev)]
        tm = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        seg_cnt = torch.zeros((args.batch, max_segs), dtype=torch.int32, device=dev)      # every segment selected for the first time
        B.thinkv_tbe_plan(gc, 0, *p_in, 10 ** 9, 256, *p_out, seg_count=seg_cnt)
        for a_, b_ in tm:
            seg_cnt.zero_()
            a_.record()
            B.thinkv_tbe_plan(gc, 0, *p_in, 10 ** 9, 256, *p_out, seg_count=seg_cnt)
            b_.record()
        torch.cuda.synchronize()
        cnts = p_out[4].cpu().numpy()
        plan = {"sequences": args.batch, "segments_per_sequence": float(n_segs.mean()), "cuts": int(cnts[0]), "tokens_listed": int(cnts[1]),
                "us_median": float(np.median([a_.elapsed_time(b_) for a_, b_ in tm]) * 1e3)}
        del p_out
    torch.cuda.synchronize()
    contrast = None
    if args.contrast:
        contrast = gather_contrast(args, np, torch, B, dev, g,
                                   lambda j: decode(gcs[j % len(gcs)], 0, q_all[nsteps - 1], out, lse, ev_seq, t_pos[nsteps - 1], 0, scale, max_ctx_pages))
    # what the memory system gives for this layout: the same (page, kv-head) blocks read by a kernel that does nothing else
    chk = torch.zeros(1, dtype=torch.int32, device=dev)
    pm = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for j in range(3):
        B.thinkv_probe_stream_pages(gcs[j % len(gcs)], 0, ev_seq, chk)
    for j, (a_, b_) in enumerate(pm):
        a_.record()
        B.thinkv_probe_stream_pages(gcs[j % len(gcs)], 0, ev_seq, chk)
        b_.record()
    torch.cuda.synchronize()
    probe_us = float(np.mean([a_.elapsed_time(b_) for a_, b_ in pm]) * 1e3)
    attn_sparsity_us = float(np.median([a.elapsed_time(b) for a, b in smarks]) * 1e3) if (args.variant == "fast" and args.format == "int") else None
    evict_us = float(np.median([m[0].elapsed_time(m[1]) for m in marks]) * 1e3)
    append_us = float(np.median([m[1].elapsed_time(m[2]) for m in marks]) * 1e3)
    evict_append_us = float(np.median([a.elapsed_time(b) for a, b in fmarks]) * 1e3)
    for gc_r in gcs:
        assert int(gc_r.dev_status.abs().sum().item()) == 0, "device flags set during the timed steps"

    # ---- algorithmic bytes of one step (from the tables as they stand after the run)
    live_by_class = []
    sm = (gc.slot_mask[:, 0] & 0xFFFF).cpu().numpy().astype(np.uint16)        # [seq][type][list position]
    npg = gc.n_pages[:, 0].cpu().numpy()
    for c in range(3):
        live_by_class.append(int(sum(np.unpackbits(sm[s, c, :npg[s, c]].view(np.uint8)).sum() for s in range(args.batch))))
    pages_visited = int(gc.n_pages[:, 0].sum().item())
    H, D, Hq = g.n_kv_heads, g.head_dim, g.n_q_heads
    kv_bytes = sum(n * H * tb for n, tb in zip(live_by_class, tok_bytes))
    attn_bytes = kv_bytes + pages_visited * 8 + args.batch * Hq * D * (2 + 2)
    append_bytes = args.batch * (2 * H * D * 2 + H * 2 * (D * 4 // 8 + D // 32 * 4) + 12)
    step_bytes = attn_bytes + append_bytes + args.batch * 12
    attn_s = float(attn_ms.mean()) * 1e-3
    achieved = attn_bytes / attn_s / 1e9
    page_bytes_read = sum(int(gc.n_pages[:, 0, c].sum().item()) * gc.page_bytes[c] for c in range(3))     # whole pages, dead slots included
    ceiling = page_bytes_read / (probe_us * 1e-6) / 1e9
    line = {
        "metric": "hybrid-quant paged decode attn: \u00b5s/step + HBM GB/s (% of peak) at 32k ctx",
        "value": step_bytes / (ms_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "us_per_step": ms_step * 1e3, "attn_us_mean": float(attn_ms.mean() * 1e3), "attn_us_min": float(attn_ms.min() * 1e3),
        "attn_us_median": float(np.median(attn_ms) * 1e3), "evict_us_median": evict_us, "append_us_median": append_us, "evict_append_us_median": evict_append_us,
        "attn_with_sparsity_statistic_us_median": attn_sparsity_us, "tbe_select": tbe, "tbe_plan": plan, "bulk_append": bulk,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16" if (args.variant == "fast" and args.format == "int") else "f32",
        "data": "synthetic",
        "config": {"workload": wl.name + f" (R1-Llama-8B layer: 32 q / 8 kv heads, head_dim 128, bf16; T{bits[0]}/R{bits[2]}/E{bits[1]}, 30% E + 10% R evicted and refilled)",
                   "batch": args.batch, "live_tokens_per_seq": int(sum(live_by_class) / args.batch), "page_size": 16,
                   "live_by_class_TER": live_by_class, "kernel": args.variant, "format": args.format, "build_seconds": round(build_s, 1), "cache_replicas": len(gcs),
                   "step": "evict 1 + append 1 (one call, thinkv_evict_append) + decode attention, per sequence"},
        "roofline": {"bound": "hbm", "kernel": "decode attention (split-K kernel + merge)", "achieved": achieved, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": achieved * 1e9 / HBM_PEAK,
                     "traffic": TRAFFIC_DEFAULT_BYTES if (args.ctx == 32768 and args.batch == 16 and args.variant == "fast" and bits == (8, 2, 4) and args.format == "int") else None,
                     "traffic_source": TRAFFIC_SOURCE, "algorithmic_bytes_per_launch": attn_bytes,
                     "stream_ceiling": {"GB/s": ceiling, "us": probe_us, "bytes": page_bytes_read, "frac_of_peak": ceiling * 1e9 / HBM_PEAK,
                                        "what": "the pages of the same launch read by a kernel that only loads (thinkv_probe_stream_pages)"},
                     "frac_of_stream_ceiling": achieved / ceiling},
        "host_wall_ms_per_step": wall / args.steps * 1e3,
    }
    if contrast is not None:
        line["gather_compaction_contrast"] = contrast
    if args.copy_calibration:
        # 2^28 int16 elements: reads 512 MiB, writes 512 MiB per call, in an elementwise kernel
        # whose name (a unary functor on short) no other kernel of this run shares
        src = torch.ones(1 << 28, dtype=torch.int16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, args, nsteps, ev_handles, new_cls, np, torch, synth)
    print(json.dumps(line))


def gather_contrast(args, np, torch, B, dev, g, attention):
    """What eviction costs when the cache is kept contiguous (Sec. 5.1 of the paper, its Observations on gather-based
    compaction): after an eviction the survivors of every sequence are gathered into a dense buffer.  Here: a binary16
    cache [batch * ctx][Hkv * D] for K and for V, 30 % of the tokens of every sequence evicted, the rest gathered row by
    row by thinkv_gather_rows (2 x Hkv * D * 2 bytes per token).  Timed alone (the sequential variant: the step waits
    for it), and looping on a second stream of the same priority while decode attention over the quantised paged cache
    runs on the first (the overlapped variant)."""
    n_tok, row = args.batch * args.ctx, g.n_kv_heads * g.head_dim
    gen = torch.Generator(device=dev).manual_seed(5)
    kv = [torch.empty((n_tok, row), dtype=torch.float16, device=dev).normal_(generator=gen) for _ in range(2)]
    keep = torch.rand(n_tok, device=dev, generator=gen) >= 0.3
    rows = torch.nonzero(keep).flatten().to(torch.int32)
    dst = [torch.empty((int(rows.numel()), row), dtype=torch.float16, device=dev) for _ in range(2)]

    def gather(stream=None):
        for a, b in zip(kv, dst):
            B.thinkv_gather_rows(a, b, rows, stream=stream)

    def timed(fn, n, stream=None):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for j, (a, b) in enumerate(ev):
            a.record(stream)
            fn(j)
            b.record(stream)
        return ev

    def med(ev):
        return float(np.median([a.elapsed_time(b) for a, b in ev]) * 1e3)

    for j in range(3):
        gather()
        attention(j)
    torch.cuda.synchronize()
    assert torch.equal(dst[0][:1000], kv[0][rows[:1000].long()])
    g_alone = timed(lambda j: gather(), 10)
    a_alone = timed(attention, 30)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g_beside = timed(lambda j: gather(side), 40, side)           # about 40 x the time of one attention call each
    a_beside = timed(attention, 60)                               # all of them start while the gathers are still running
    still_running = not g_beside[-1][1].query()
    torch.cuda.synchronize()
    moved = 2 * int(rows.numel()) * row * 2 * 2               # read + written
    ga, aa, gb, ab = med(g_alone), med(a_alone), med(g_beside), med(a_beside)
    return {"contiguous_f16_cache_GB": 2 * n_tok * row * 2 / 1e9, "evicted_fraction": 0.3, "bytes_moved_per_compaction": moved,
            "gather_kernel": "thinkv_gather_rows",
            "gather_us_alone": ga, "gather_GB_per_s_alone": moved / ga / 1e3, "attention_us_alone": aa,
            "attention_us_beside_gather": ab, "attention_slowdown_beside_gather": ab / aa, "gather_us_beside_attention": gb,
            "gathers_outlasted_the_attention_calls": bool(still_running),
            "step_us_if_compacted_every_step_sequential": ga + aa, "slowdown_if_compacted_every_step": (ga + aa) / aa,
            "in_place_reuse_bytes_moved": 0}


def e2e_cfg5(args, np, torch, B, synth, harness, dev):
    """Configuration 5 as written: the ragged batch of 256 (contexts log-uniform in 1k..64k) is bulk-built on `--layers`
    layers of the 8B shape, then 64 consecutive decode steps run; a step appends one token per sequence on every layer,
    every 16th step begins with an eviction pass that removes 5 % of the live tokens of the least important class (E,
    seeded uniform choice per sequence and layer), and runs decode attention on every layer."""
    n_steps, L = 64, args.layers
    g = synth.Geometry(L, 32, 8, 128, "bf16")
    ctx = synth.stress_contexts(4, 256)
    wl = synth.stress_decode("cfg5-stress-8b", g, 4, ctx, 0)
    S = wl.n_seqs
    t0 = time.time()
    need = np.array(harness.arena_need(wl, slack=1.0), dtype=np.int64)
    arena = tuple(int(x * 1.03) + S * L * 8 for x in need)
    gc = harness.make_gpu_cache(wl, arena_pages=arena, max_pages=harness.max_pages_need(wl) + 8)
    gr = synth.ScriptRunner(wl, harness.GpuBackend(gc)).run()
    torch.cuda.synchronize()
    build_s = time.time() - t0
    assert int(gc.dev_status.abs().sum().item()) == 0, "device flags set while building the cache"
    # ---- inputs of the steps, resident before timing starts
    gen = torch.Generator(device=dev).manual_seed(99)
    rng = np.random.default_rng(99)
    scale_ch = torch.ones(g.head_dim, device=dev)
    scale_ch[list(synth.outlier_channels(g.head_dim))] = 8.0
    kv_new = [(torch.randn((n_steps, S, g.n_kv_heads, g.head_dim), device=dev, generator=gen) * scale_ch).to(torch.bfloat16) for _ in range(2 * L)]
    q = [torch.randn((S, g.n_q_heads, g.head_dim), device=dev, generator=gen).to(torch.bfloat16) for _ in range(L)]
    new_cls = np.stack([synth.thought_classes(rng, n_steps)[0] for _ in range(S)], 1)          # [step][seq]
    t_cls = torch.from_numpy(new_cls).to(dev)
    t_pos = torch.from_numpy(np.stack([ctx + st for st in range(n_steps)]).astype(np.int32)).to(dev)
    seqs = torch.arange(S, dtype=torch.int32, device=dev)
    ev_lists = {}
    for l in range(L):
        cand = [np.flatnonzero(wl.classes[s_][:ctx[s_]] == synth.E) for s_ in range(S)]
        for p_ in range(n_steps // 16):
            es, eh = [], []
            for s_ in range(S):
                n = int(round(0.05 * len(cand[s_])))
                if n == 0:
                    continue
                pick = rng.choice(len(cand[s_]), size=n, replace=False)
                eh.append(gr.handle[(l, s_)][cand[s_][pick]])
                es.append(np.full(n, s_, np.int32))
                cand[s_] = np.delete(cand[s_], pick)
            ev_lists[(l, p_)] = (torch.from_numpy(np.concatenate(es)).to(dev), torch.from_numpy(np.concatenate(eh).astype(np.int32)).to(dev))
    out = torch.empty((S, g.n_q_heads, g.head_dim), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((S, g.n_q_heads), dtype=torch.float32, device=dev)
    h_out = torch.empty(S, dtype=torch.int32, device=dev)
    mcp = [int(gc.n_pages[:, l].sum(-1).max().item()) + n_steps // 16 + 4 for l in range(L)]
    scale = g.head_dim ** -0.5

    def step(st, marks=None):
        for l in range(L):
            if marks is not None:
                marks[l][0].record()
            if st % 16 == 15:
                B.thinkv_evict(gc, l, *ev_lists[(l, st // 16)])
            if marks is not None:
                marks[l][1].record()
            B.thinkv_append_quantized(gc, l, kv_new[2 * l][st], kv_new[2 * l + 1][st], seqs, t_pos[st], t_cls[st], h_out)
            if marks is not None:
                marks[l][2].record()
            B.thinkv_decode_attention(gc, l, q[l], out, lse, seqs, t_pos[st], 0, scale, mcp[l])
            if marks is not None:
                marks[l][3].record()

    marks = [[[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(L)] for _ in range(n_steps)]
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)]
    torch.cuda.synchronize()
    step_ev[0].record()
    for st in range(n_steps):
        step(st, marks[st])
        step_ev[st + 1].record()
    torch.cuda.synchronize()
    assert int(gc.dev_status.abs().sum().item()) == 0, "device flags set during the steps"
    step_ms = np.array([step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(n_steps)])
    ev_us = np.array([[m[0].elapsed_time(m[1]) * 1e3 for m in marks[st]] for st in range(n_steps)])
    ap_us = np.array([[m[1].elapsed_time(m[2]) * 1e3 for m in marks[st]] for st in range(n_steps)])
    at_us = np.array([[m[2].elapsed_time(m[3]) * 1e3 for m in marks[st]] for st in range(n_steps)])
    # algorithmic bytes of a step, from the tables as they stand at the end
    H, D, Hq = g.n_kv_heads, g.head_dim, g.n_q_heads
    live_by_class = [0, 0, 0]
    for l in range(L):
        sm = (gc.slot_mask[:, l] & 0xFFFF).cpu().numpy().astype(np.uint16)
        npg = gc.n_pages[:, l].cpu().numpy()
        for c in range(3):
            live_by_class[c] += int(sum(np.unpackbits(sm[s_, c, :npg[s_, c]].view(np.uint8)).sum() for s_ in range(S)))
    kv_bytes = sum(n * H * 2 * (D * b // 8 + D // 32 * 4) for n, b in zip(live_by_class, g.bits_of_class))
    attn_bytes = kv_bytes + int(gc.n_pages.sum().item()) * 8 + L * S * Hq * D * 4
    append_bytes = L * S * (2 * H * D * 2 + H * 2 * (D * 4 // 8 + D // 32 * 4) + 12)
    ms = float(step_ms.mean())
    line = {
        "metric": "hybrid-quant paged decode attn: \u00b5s/step + HBM GB/s (% of peak) at 32k ctx",
        "value": (attn_bytes + append_bytes) / (ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": n_steps, "warmup": 0,
        "ms_per_step": ms, "ms_per_step_min": float(step_ms.min()), "ms_per_step_with_eviction_pass": float(step_ms[15::16].mean()),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "cfg5 as written: ragged batch 256 (contexts log-uniform 1k..64k), 8B shape, 64 consecutive decode steps",
                   "layers_built": L, "layers_of_the_configuration": 32, "scaled_down": L != 32, "batch": S,
                   "live_tokens_per_layer": int(sum(live_by_class) / L), "build_seconds": round(build_s, 1),
                   "step": "per layer: [every 16th step: evict 5% of the live E tokens of every sequence] + append 1 token per sequence + decode attention"},
        "per_layer_us": {"attention_mean": float(at_us.mean()), "append_mean": float(ap_us.mean()),
                         "evict_pass_mean": float(ev_us[15::16].mean()), "attention_GB_per_s": attn_bytes / L / (float(at_us.mean()) * 1e-6) / 1e9,
                         "attention_frac_of_8TBps": attn_bytes / L / (float(at_us.mean()) * 1e-6) / HBM_PEAK},
        "algorithmic_bytes_per_step": attn_bytes + append_bytes,
    }
    if not args.no_cpu_baseline:
        # the oracle on ONE (sequence, layer) of the same workload: the sequence of median context, whole steps
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import parity
        from oracle import attention as oattn
        s_ = int(np.argsort(ctx)[S // 2])
        ob = parity.make_oracle(wl, max_seqs=S, arena_pages=tuple(int(x) + 16 for x in harness.arena_need_one(wl, s_)))
        synth.ScriptRunner(wl, ob, layers=[0], seqs=[s_]).run()
        oc = ob.cache
        cpu = torch.device("cpu")
        k1 = kv_new[0][:, s_].float().cpu().numpy()
        v1 = kv_new[1][:, s_].float().cpu().numpy()
        q1 = q[0][s_].float().cpu().numpy().astype(np.float64)[None]
        t1 = time.perf_counter()
        done = 0
        while done < n_steps and (done < 1 or time.perf_counter() - t1 < args.cpu_seconds):
            oc.append(0, k1[done:done + 1], v1[done:done + 1], [s_], [int(ctx[s_]) + done], [new_cls[done, s_]])
            oattn.decode_attention(oc, 0, q1, [s_], [int(ctx[s_]) + done], 0, scale)
            done += 1
        dt = (time.perf_counter() - t1) / done
        line["cpu_baseline"] = {"value": oc.stored_bytes_live(s_, 0) / dt / 1e9, "unit": "GB/s", "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
                                "seconds_per_sequence_layer_step": dt,
                                "sample": f"{done} steps (append 1, binary64 attention) of one sequence (context {int(ctx[s_])}, the batch's median) on one layer; "
                                          f"a whole step is {S} sequences x {L} layers of this"}
    return line


def attention_only(args, np, torch, B, synth, harness, dev):
    """Decode attention alone on one of the other configurations: the cache is built by the
    configuration's own script (bulk append, eviction, refill or budgeted decode), then a step is
    one attention call per built layer for the whole batch."""
    wl = {"cfg1": lambda: synth.config_tiny(),
          "cfg2": lambda: synth.config_llama8b_layer(seed=1, n_seqs=16, ctx=8192, refill_chunk=64),
          "cfg3": lambda: synth.config_qwen14b_budget(),
          "cfg4": lambda: synth.config_gptoss(n_layers=4),
          "cfg5": lambda: synth.config_stress(n_layers=2, n_steps=32)}[args.workload]()
    g = wl.geom
    t0 = time.time()
    gc = harness.make_gpu_cache(wl)
    synth.ScriptRunner(wl, harness.GpuBackend(gc)).run()
    torch.cuda.synchronize()
    assert int(gc.dev_status.abs().sum().item()) == 0, "device flags set while building the cache"
    # Copies of the cache to rotate over, so that a call does not find its pages in the 256 MB
    # memory-side cache from the call before: enough for 1 GB in all, at most four.
    stored = sum(int(gc.n_pages[:, :, c].sum().item()) * gc.page_bytes[c] for c in range(3))
    n_rep = int(min(4, max(1, -(-(1 << 30) // max(stored, 1)))))
    gcs = [gc]
    for _ in range(n_rep - 1):
        gcs.append(harness.make_gpu_cache(wl))
        synth.ScriptRunner(wl, harness.GpuBackend(gcs[-1])).run()
    torch.cuda.synchronize()
    build_s = time.time() - t0
    L, S = g.n_layers, wl.n_seqs
    q = [torch.stack([synth.query_rows(wl.seed, l, s_, 0, g, dev) for s_ in range(S)]).contiguous() for l in range(L)]
    out = torch.empty(q[0].shape, dtype=q[0].dtype, device=dev)
    lse = torch.empty((S, g.n_q_heads), dtype=torch.float32, device=dev)
    sid = torch.arange(S, dtype=torch.int32, device=dev)
    qp = torch.from_numpy(wl.q_pos.astype(np.int32)).to(dev)
    mcp = [int(gc.n_pages[:, l].sum(-1).max().item()) for l in range(L)]
    scale = g.head_dim ** -0.5

    def step(i, marks=None, rotate=True):
        c_ = gcs[i % len(gcs)] if rotate else gcs[0]
        for l in range(L):
            if marks is not None:
                marks[l][0].record()
            B.thinkv_decode_attention(c_, l, q[l], out, lse, sid, qp, wl.window_of_layer[l], scale, mcp[l])
            if marks is not None:
                marks[l][1].record()

    def new_marks():
        return [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)] for _ in range(args.steps)]

    for i in range(args.warmup):
        step(i)
    marks = new_marks()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(args.steps):
        step(i, marks[i])
    e1.record()
    torch.cuda.synchronize()
    ms_step = e0.elapsed_time(e1) / args.steps
    per_layer_us = np.array([[a.elapsed_time(b) * 1e3 for a, b in m] for m in marks])     # [steps][layers]
    # the same on one copy only ("hot": what fits stays in the memory-side cache between calls)
    hot = new_marks()
    for i in range(args.steps):
        step(i, hot[i], rotate=False)
    torch.cuda.synchronize()
    hot_us = np.median(np.array([[a.elapsed_time(b) * 1e3 for a, b in m] for m in hot]), axis=0)
    # algorithmic bytes per layer: live tokens visible to the query, page ids + masks, q and out
    H, D, Hq = g.n_kv_heads, g.head_dim, g.n_q_heads
    npg = gc.n_pages.cpu().numpy()
    sm = (gc.slot_mask & 0xFFFF).cpu().numpy().astype(np.uint16)
    layer_bytes, layer_live = [], []
    for l in range(L):
        W = wl.window_of_layer[l]
        tot, live_l = 0, 0
        for c in range(3):
            tok_b = H * 2 * (D * g.bits_of_class[c] // 8 + D // 32 * 4)
            if W == 0:
                n = int(sum(np.unpackbits(sm[s_, l, c, :npg[s_, l, c]].view(np.uint8)).sum() for s_ in range(S)))
            else:
                pos = gc.slot_pos[c].cpu().numpy()
                n = 0
                for s_ in range(S):
                    ids = gc.block_table[s_, l, c, :npg[s_, l, c]].cpu().numpy()
                    m = np.unpackbits(sm[s_, l, c, :npg[s_, l, c]].view(np.uint8).reshape(-1, 2), axis=1, bitorder="little").astype(bool)
                    d = int(wl.q_pos[s_]) - pos[ids]
                    n += int((m & (d >= 0) & (d < W)).sum())
            tot += n * tok_b
            live_l += n
        pages = int(npg[:, l].sum())
        tot += pages * (8 + (64 if W else 0)) + S * Hq * D * (2 + q[0].element_size())
        layer_bytes.append(tot)
        layer_live.append(live_l)
    med = np.median(per_layer_us, axis=0)
    return {
        "metric": "hybrid-quant paged decode attn: \u00b5s/step + HBM GB/s (% of peak) at 32k ctx",
        "value": sum(layer_bytes) / (ms_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": wl.name, "batch": S, "layers_built": L, "window_of_layer": list(wl.window_of_layer),
                   "step": "decode attention alone, one call per built layer", "build_seconds": round(build_s, 1),
                   "cache_replicas": len(gcs), "stored_bytes_per_replica": int(stored),
                   "live_tokens_visible_per_layer": layer_live},
        "per_layer": [{"layer": l, "window": int(wl.window_of_layer[l]), "attn_us_median": float(med[l]),
                       "attn_us_min": float(per_layer_us[:, l].min()), "attn_us_median_one_copy_hot": float(hot_us[l]),
                       "algorithmic_bytes": int(layer_bytes[l]),
                       "GB/s": layer_bytes[l] / (med[l] * 1e-6) / 1e9, "frac_of_8TBps": layer_bytes[l] / (med[l] * 1e-6) / HBM_PEAK}
                      for l in range(L)],
    }


def cpu_baseline(wl, args, nsteps, ev_handles, new_cls, np, torch, synth):
    """The oracle as it stands, timed on this machine's host cores on ONE sequence of the same
    workload (sequence 0: its full build is replayed untimed, then whole steps are timed).
    The only part of the default run that loads anything from oracle/ (through the test helpers)."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import parity
    from oracle import attention as oattn
    # the host cores this process may run on; the oracle itself is NumPy (one Python thread, BLAS
    # threads inside the matrix products)
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas_threads = None
    g = wl.geom
    ob = parity.make_oracle(wl, max_seqs=1, arena_pages=tuple(int(x) + 8 for x in parity.backends.arena_need(wl)),
                            max_pages=parity.backends.max_pages_need(wl) + 8)
    synth.ScriptRunner(wl, ob, seqs=[0]).run()
    oc = ob.cache
    n0 = len(wl.classes[0])
    cpu = torch.device("cpu")
    k = synth.kv_rows(wl.seed, 0, 0, 0, n0, n0 + nsteps, g, cpu).float().numpy()
    v = synth.kv_rows(wl.seed, 0, 0, 1, n0, n0 + nsteps, g, cpu).float().numpy()
    t0 = time.perf_counter()
    done = 0
    live = 0
    t_ev = t_ap = t_at = 0.0
    while done < nsteps and (done < 1 or time.perf_counter() - t0 < args.cpu_seconds):
        i = done
        ta = time.perf_counter()
        oc.evict_slots(0, [0], [ev_handles[i, 0]])
        tb = time.perf_counter()
        oc.append(0, k[i:i + 1], v[i:i + 1], [0], [n0 + i], [new_cls[i, 0]])
        tc = time.perf_counter()
        q = synth.query_rows(wl.seed, 0, 0, i, g, cpu).float().numpy().astype(np.float64)[None]
        oattn.decode_attention(oc, 0, q, [0], [n0 + i], 0, g.head_dim ** -0.5)
        td = time.perf_counter()
        t_ev, t_ap, t_at = t_ev + tb - ta, t_ap + tc - tb, t_at + td - tc
        live = oc.stored_bytes_live(0, 0)
        done += 1
    dt = time.perf_counter() - t0
    return {"value": live * done / dt / 1e9, "unit": "GB/s", "cores": cores, "blas_threads": blas_threads, "kind": "oracle",
            "seconds_per_sequence_step": dt / done,
            "us_per_sequence_evict_1": t_ev / done * 1e6, "us_per_sequence_append_1": t_ap / done * 1e6,
            "us_per_sequence_attention": t_at / done * 1e6,
            "sample": f"{done} whole steps (evict 1, append 1, binary64 attention) of sequence 0 of the same workload "
                      f"({int(oc.n_live[0, 0])} live tokens); a batch step costs {args.batch}x this"}


if __name__ == "__main__":
    main()
