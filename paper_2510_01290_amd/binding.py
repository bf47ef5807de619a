"""ctypes binding of libthinkv.so (include/thinkv.h).  Argument marshalling only: every step
of the path runs in the HIP kernels; torch supplies device memory and the current stream.
There is no CPU fallback: a missing library raises."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libthinkv.so")
_lib = None

F16, BF16, F32 = 0, 1, 2
_DT = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}
ST_NOPAGES, ST_BAD_CLASS, ST_BAD_SLOT, ST_EVICT_DEAD, ST_BAD_SEQ, ST_BAD_SEGMENT = 1, 2, 4, 8, 16, 32
EXPORTS = ["thinkv_block_bytes", "thinkv_page_bytes", "thinkv_append_workspace_bytes",
           "thinkv_decode_workspace_bytes", "thinkv_init_view", "thinkv_append_quantized", "thinkv_evict", "thinkv_evict_append",
           "thinkv_decode_attention", "thinkv_decode_attention_noalloc", "thinkv_decode_attention_valu", "thinkv_decode_sparsity_workspace_bytes",
           "thinkv_decode_attention_sparsity", "thinkv_tbe_workspace_bytes", "thinkv_tbe_select", "thinkv_tbe_plan_workspace_bytes", "thinkv_tbe_plan", "thinkv_probe_stream_pages", "thinkv_gather_rows",
           "thinkv_status_string"]


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("group_size", C.c_int32),
                ("bits_of_class", C.c_int32 * 3), ("max_seqs", C.c_int32), ("max_pages", C.c_int32),
                ("format", C.c_int32), ("fp8_scale", C.c_float * 2)]


class View(C.Structure):
    _fields_ = [("cfg", Config), ("arena", C.c_void_p * 3), ("arena_pages", C.c_int64 * 3),
                ("free_stack", C.c_void_p * 3), ("free_top", C.c_void_p), ("block_table", C.c_void_p),
                ("n_pages", C.c_void_p), ("page_filled", C.c_void_p * 3), ("slot_mask", C.c_void_p),
                ("slot_pos", C.c_void_p * 3), ("page_pos_max", C.c_void_p * 3), ("n_live", C.c_void_p), ("work_counters", C.c_void_p), ("append_counters", C.c_void_p),
                ("dev_status", C.c_void_p)]


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python __graft_entry__.py` (hipcc, gfx950)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.thinkv_block_bytes.restype = sz
    lib.thinkv_block_bytes.argtypes = [C.POINTER(Config), C.c_int]
    lib.thinkv_page_bytes.restype = sz
    lib.thinkv_page_bytes.argtypes = [C.POINTER(Config), C.c_int]
    lib.thinkv_append_workspace_bytes.restype = sz
    lib.thinkv_append_workspace_bytes.argtypes = [C.POINTER(Config), i32]
    lib.thinkv_decode_workspace_bytes.restype = sz
    lib.thinkv_decode_workspace_bytes.argtypes = [C.POINTER(Config), i32, i32]
    lib.thinkv_init_view.restype = C.c_int
    lib.thinkv_init_view.argtypes = [C.POINTER(View), vp]
    lib.thinkv_append_quantized.restype = C.c_int
    lib.thinkv_append_quantized.argtypes = [C.POINTER(View), i32, vp, vp, vp, vp, vp, vp, i32, C.c_int, vp, sz, vp]
    lib.thinkv_evict.restype = C.c_int
    lib.thinkv_evict.argtypes = [C.POINTER(View), i32, vp, vp, i32, vp]
    lib.thinkv_evict_append.restype = C.c_int
    lib.thinkv_evict_append.argtypes = [C.POINTER(View), i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, i32, C.c_int, vp, sz, vp]
    for name in ("thinkv_decode_attention", "thinkv_decode_attention_valu"):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [C.POINTER(View), i32, vp, vp, vp, vp, vp, i32, i32, C.c_float, C.c_int, C.c_int, i32, vp, sz, vp]
    lib.thinkv_decode_attention_noalloc.restype = C.c_int
    lib.thinkv_decode_attention_noalloc.argtypes = [C.POINTER(View), i32, vp, vp, vp, vp, vp, i32, i32, C.c_float, C.c_int, C.c_int, i32, vp]
    lib.thinkv_decode_sparsity_workspace_bytes.restype = sz
    lib.thinkv_decode_sparsity_workspace_bytes.argtypes = [C.POINTER(Config), i32, i32]
    lib.thinkv_decode_attention_sparsity.restype = C.c_int
    lib.thinkv_decode_attention_sparsity.argtypes = [C.POINTER(View), i32, vp, vp, vp, vp, vp, vp, i32, i32, C.c_float, C.c_int, C.c_int,
                                                     i32, vp, sz, vp]
    lib.thinkv_tbe_workspace_bytes.restype = sz
    lib.thinkv_tbe_workspace_bytes.argtypes = [C.POINTER(Config), i32, i32]
    lib.thinkv_tbe_select.restype = C.c_int
    lib.thinkv_tbe_select.argtypes = [C.POINTER(View), i32, vp, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
    lib.thinkv_tbe_plan_workspace_bytes.restype = sz
    lib.thinkv_tbe_plan_workspace_bytes.argtypes = [i32, i32]
    lib.thinkv_tbe_plan.restype = C.c_int
    lib.thinkv_tbe_plan.argtypes = [C.POINTER(View), i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.thinkv_probe_stream_pages.restype = C.c_int
    lib.thinkv_probe_stream_pages.argtypes = [C.POINTER(View), i32, vp, i32, vp, vp]
    lib.thinkv_gather_rows.restype = C.c_int
    lib.thinkv_gather_rows.argtypes = [vp, vp, vp, C.c_int64, i32, vp]
    lib.thinkv_status_string.restype = C.c_char_p
    lib.thinkv_status_string.argtypes = [C.c_int]
    _lib = lib
    return lib


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what}: {load().thinkv_status_string(rc).decode()} (status {rc})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


FMT_INT, FMT_FP = 0, 1


def make_config(n_layers, n_q_heads, n_kv_heads, head_dim, bits_of_class, max_seqs, max_pages, fmt=FMT_INT, fp8_scale=(1.0, 1.0)):
    return Config(n_layers, n_q_heads, n_kv_heads, head_dim, 16, 32, (C.c_int32 * 3)(*bits_of_class), max_seqs, max_pages,
                  fmt, (C.c_float * 2)(*fp8_scale))


def thinkv_block_bytes(cfg, bits):
    return load().thinkv_block_bytes(C.byref(cfg), bits)


def thinkv_page_bytes(cfg, bits):
    return load().thinkv_page_bytes(C.byref(cfg), bits)


def thinkv_append_workspace_bytes(cfg, n_tok):
    return load().thinkv_append_workspace_bytes(C.byref(cfg), n_tok)


def thinkv_decode_workspace_bytes(cfg, B, max_ctx_pages):
    return load().thinkv_decode_workspace_bytes(C.byref(cfg), B, max_ctx_pages)


class Cache:
    """Device buffers of one cache (torch tensors) and the thinkv_view that points at them."""

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, bits_of_class, max_seqs, max_pages,
                 arena_pages, device="cuda:0", fmt=FMT_INT, fp8_scale=(1.0, 1.0)):
        load()
        self.device = torch.device(device)
        self.cfg = make_config(n_layers, n_q_heads, n_kv_heads, head_dim, bits_of_class, max_seqs, max_pages, fmt, fp8_scale)
        self.bits_of_class = tuple(bits_of_class)
        self.arena_pages = tuple(int(x) for x in arena_pages)
        d = self.device
        self.page_bytes = [thinkv_page_bytes(self.cfg, b) for b in bits_of_class]
        if 0 in self.page_bytes:
            raise RuntimeError("unsupported geometry")
        self.arena = [torch.empty(max(1, n) * pb, dtype=torch.uint8, device=d) for n, pb in zip(self.arena_pages, self.page_bytes)]
        self.free_stack = [torch.empty(max(1, n), dtype=torch.int32, device=d) for n in self.arena_pages]
        self.free_top = torch.empty(3, dtype=torch.int32, device=d)
        self.block_table = torch.empty((max_seqs, n_layers, 3, max_pages), dtype=torch.int32, device=d)
        self.n_pages = torch.empty((max_seqs, n_layers, 3), dtype=torch.int32, device=d)
        self.page_filled = [torch.empty(max(1, n), dtype=torch.uint8, device=d) for n in self.arena_pages]
        self.slot_mask = torch.empty((max_seqs, n_layers, 3, max_pages), dtype=torch.int32, device=d)
        self.slot_pos = [torch.empty((max(1, n), 16), dtype=torch.int32, device=d) for n in self.arena_pages]
        self.page_pos_max = [torch.empty(max(1, n), dtype=torch.int32, device=d) for n in self.arena_pages]
        self.n_live = torch.empty((max_seqs, n_layers), dtype=torch.int32, device=d)
        self.work_counters = torch.empty((n_layers, max_seqs, n_kv_heads, 4), dtype=torch.int32, device=d)
        self.append_counters = torch.empty(max_seqs, dtype=torch.int32, device=d)
        self.dev_status = torch.empty(max_seqs * n_layers + 1, dtype=torch.int32, device=d)
        v = View()
        v.cfg = self.cfg
        for k in range(3):
            v.arena[k] = self.arena[k].data_ptr()
            v.arena_pages[k] = self.arena_pages[k]
            v.free_stack[k] = self.free_stack[k].data_ptr()
            v.page_filled[k] = self.page_filled[k].data_ptr()
            v.slot_pos[k] = self.slot_pos[k].data_ptr()
            v.page_pos_max[k] = self.page_pos_max[k].data_ptr()
        v.free_top = self.free_top.data_ptr()
        v.block_table = self.block_table.data_ptr()
        v.slot_mask = self.slot_mask.data_ptr()
        v.n_pages = self.n_pages.data_ptr()
        v.n_live = self.n_live.data_ptr()
        v.work_counters = self.work_counters.data_ptr()
        v.append_counters = self.append_counters.data_ptr()
        v.dev_status = self.dev_status.data_ptr()
        self.view = v
        self._ws = None
        thinkv_init_view(self)

    def workspace(self, nbytes):
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(int(nbytes * 1.25) + 256, dtype=torch.uint8, device=self.device)
        return self._ws


def thinkv_init_view(cache, stream=None):
    _check(load().thinkv_init_view(C.byref(cache.view), _stream(stream)), "thinkv_init_view")


def thinkv_append_quantized(cache, layer, k_new, v_new, tok_seq, tok_pos, tok_class, tok_handle=None, stream=None):
    """k_new, v_new: [n_tok, Hkv, D] device tensors (f16/bf16/f32, contiguous); tok_seq/tok_pos int32,
    tok_class uint8, tok_handle int32 (optional, out) device tensors."""
    n_tok = int(tok_seq.numel())
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == v_new.dtype
    assert tok_seq.dtype == torch.int32 and tok_pos.dtype == torch.int32 and tok_class.dtype == torch.uint8
    assert tuple(k_new.shape) == (n_tok, cache.cfg.n_kv_heads, cache.cfg.head_dim) == tuple(v_new.shape)
    nb = thinkv_append_workspace_bytes(cache.cfg, n_tok)
    ws = cache.workspace(nb)
    _check(load().thinkv_append_quantized(C.byref(cache.view), layer, _ptr(k_new), _ptr(v_new), _ptr(tok_seq),
                                          _ptr(tok_pos), _ptr(tok_class), _ptr(tok_handle), n_tok, _DT[k_new.dtype],
                                          _ptr(ws), ws.numel(), _stream(stream)), "thinkv_append_quantized")


def thinkv_evict_append(cache, layer, ev_seq, ev_handle, k_new, v_new, tok_seq, tok_pos, tok_class, tok_handle=None, stream=None):
    """thinkv_evict followed by thinkv_append_quantized, in one call"""
    n_tok = int(tok_seq.numel())
    assert ev_seq.dtype == torch.int32 and ev_handle.dtype == torch.int32 and ev_seq.numel() == ev_handle.numel()
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == v_new.dtype
    assert tok_seq.dtype == torch.int32 and tok_pos.dtype == torch.int32 and tok_class.dtype == torch.uint8
    assert tuple(k_new.shape) == (n_tok, cache.cfg.n_kv_heads, cache.cfg.head_dim) == tuple(v_new.shape)
    nb = thinkv_append_workspace_bytes(cache.cfg, n_tok)
    ws = cache.workspace(nb)
    _check(load().thinkv_evict_append(C.byref(cache.view), layer, _ptr(ev_seq), _ptr(ev_handle), int(ev_seq.numel()),
                                      _ptr(k_new), _ptr(v_new), _ptr(tok_seq), _ptr(tok_pos), _ptr(tok_class), _ptr(tok_handle),
                                      n_tok, _DT[k_new.dtype], _ptr(ws), ws.numel(), _stream(stream)), "thinkv_evict_append")


def thinkv_evict(cache, layer, ev_seq, ev_handle, stream=None):
    assert ev_seq.dtype == torch.int32 and ev_handle.dtype == torch.int32
    _check(load().thinkv_evict(C.byref(cache.view), layer, _ptr(ev_seq), _ptr(ev_handle), int(ev_seq.numel()),
                               _stream(stream)), "thinkv_evict")


def _decode(fn, cache, layer, q, out, lse, seq_ids, q_pos, window, softmax_scale, max_ctx_pages, stream):
    B = int(q.shape[0])
    assert q.is_contiguous() and out.is_contiguous() and tuple(q.shape) == tuple(out.shape)
    assert tuple(q.shape[1:]) == (cache.cfg.n_q_heads, cache.cfg.head_dim)
    assert seq_ids.dtype == torch.int32 and (q_pos is None or q_pos.dtype == torch.int32)
    assert lse is None or (lse.dtype == torch.float32 and lse.numel() == B * cache.cfg.n_q_heads)
    nb = thinkv_decode_workspace_bytes(cache.cfg, B, max_ctx_pages)
    ws = cache.workspace(nb)
    _check(fn(C.byref(cache.view), layer, _ptr(q), _ptr(out), _ptr(lse), _ptr(seq_ids), _ptr(q_pos), B, window,
              float(softmax_scale), _DT[q.dtype], _DT[out.dtype], int(max_ctx_pages), _ptr(ws), ws.numel(),
              _stream(stream)), "thinkv_decode_attention")


def thinkv_decode_attention(cache, layer, q, out, lse, seq_ids, q_pos, window, softmax_scale, max_ctx_pages, stream=None):
    _decode(load().thinkv_decode_attention, cache, layer, q, out, lse, seq_ids, q_pos, window, softmax_scale,
            max_ctx_pages, stream)


NOALLOC_SCRATCH_BYTES = 32 << 20


def thinkv_decode_attention_noalloc(cache, layer, q, out, lse, seq_ids, q_pos, window, softmax_scale, max_ctx_pages, stream=None):
    """thinkv_decode_attention without a workspace: the partial rows live in the library's own device array"""
    B = int(q.shape[0])
    assert q.is_contiguous() and out.is_contiguous() and tuple(q.shape) == tuple(out.shape)
    assert tuple(q.shape[1:]) == (cache.cfg.n_q_heads, cache.cfg.head_dim)
    assert seq_ids.dtype == torch.int32 and (q_pos is None or q_pos.dtype == torch.int32)
    assert lse is None or (lse.dtype == torch.float32 and lse.numel() == B * cache.cfg.n_q_heads)
    _check(load().thinkv_decode_attention_noalloc(C.byref(cache.view), layer, _ptr(q), _ptr(out), _ptr(lse), _ptr(seq_ids), _ptr(q_pos), B,
                                                  window, float(softmax_scale), _DT[q.dtype], _DT[out.dtype], int(max_ctx_pages),
                                                  _stream(stream)), "thinkv_decode_attention_noalloc")


TBE_BY_COUNT, TBE_BY_SIZE = 0, 1


def thinkv_tbe_plan(cache, layer, seq_ids, seg_start, seg_type, n_segs, transition_ended, budget, max_cuts, tok_seq, tok_handle,
                    seg_offset, seg_keep, counts, seg_count=None, rule=TBE_BY_COUNT, stream=None):
    """seg_count [max_seqs, max_segs] int32 in/out (selections of every segment so far; rule TBE_BY_COUNT);
    seg_start [max_seqs, max_segs] int32, seg_type [max_seqs, max_segs] uint8, n_segs [max_seqs] int32, seq_ids [B] int32,
    transition_ended [B] uint8 or None; outputs tok_seq / tok_handle [cap_tok], seg_offset [cap_seg + 1], seg_keep [cap_seg],
    counts [2], all int32 device tensors."""
    B, max_segs = int(seq_ids.numel()), int(seg_start.shape[1])
    cap_tok, cap_seg = int(tok_handle.numel()), int(seg_keep.numel())
    assert seg_start.dtype == torch.int32 and seg_type.dtype == torch.uint8 and n_segs.dtype == torch.int32
    assert seg_start.is_contiguous() and seg_type.is_contiguous() and tuple(seg_type.shape) == tuple(seg_start.shape)
    assert tok_seq.numel() == cap_tok and seg_offset.numel() == cap_seg + 1 and counts.numel() == 2
    for t in (seq_ids, tok_seq, tok_handle, seg_offset, seg_keep, counts):
        assert t.dtype == torch.int32 and t.is_contiguous()
    assert transition_ended is None or (transition_ended.dtype == torch.uint8 and transition_ended.numel() == B)
    assert seg_count is None or (seg_count.dtype == torch.int32 and seg_count.is_contiguous() and tuple(seg_count.shape) == tuple(seg_start.shape))
    nb = load().thinkv_tbe_plan_workspace_bytes(B, int(max_cuts))
    ws = cache.workspace(nb)
    _check(load().thinkv_tbe_plan(C.byref(cache.view), layer, _ptr(seq_ids), _ptr(seg_start), _ptr(seg_type), _ptr(n_segs),
                                  _ptr(transition_ended), _ptr(seg_count), int(rule), B, max_segs, int(budget), int(max_cuts), cap_seg, cap_tok, _ptr(tok_seq),
                                  _ptr(tok_handle), _ptr(seg_offset), _ptr(seg_keep), _ptr(counts), _ptr(ws), ws.numel(),
                                  _stream(stream)), "thinkv_tbe_plan")


def thinkv_tbe_select(cache, layer, tok_seq, tok_handle, seg_offset, seg_keep, ev_handle, max_iters=8, stream=None):
    n_tok, n_seg = int(tok_handle.numel()), int(seg_keep.numel())
    for t in (tok_seq, tok_handle, seg_offset, seg_keep, ev_handle):
        assert t.dtype == torch.int32 and t.is_contiguous()
    assert tok_seq.numel() == n_tok and ev_handle.numel() == n_tok and seg_offset.numel() == n_seg + 1
    nb = load().thinkv_tbe_workspace_bytes(C.byref(cache.cfg), n_tok, n_seg)
    ws = cache.workspace(nb)
    _check(load().thinkv_tbe_select(C.byref(cache.view), layer, _ptr(tok_seq), _ptr(tok_handle), _ptr(seg_offset), _ptr(seg_keep),
                                    n_seg, n_tok, int(max_iters), _ptr(ev_handle), _ptr(ws), ws.numel(), _stream(stream)),
           "thinkv_tbe_select")


def thinkv_decode_attention_sparsity(cache, layer, q, out, lse, sparsity, seq_ids, q_pos, window, softmax_scale, max_ctx_pages,
                                     stream=None):
    B = int(q.shape[0])
    assert q.is_contiguous() and out.is_contiguous() and tuple(q.shape) == tuple(out.shape)
    assert tuple(q.shape[1:]) == (cache.cfg.n_q_heads, cache.cfg.head_dim)
    assert seq_ids.dtype == torch.int32 and (q_pos is None or q_pos.dtype == torch.int32)
    assert lse is None or (lse.dtype == torch.float32 and lse.numel() == B * cache.cfg.n_q_heads)
    assert sparsity.dtype == torch.float32 and sparsity.numel() == B and sparsity.is_contiguous()
    nb = load().thinkv_decode_sparsity_workspace_bytes(C.byref(cache.cfg), B, int(max_ctx_pages))
    ws = cache.workspace(nb)
    _check(load().thinkv_decode_attention_sparsity(
        C.byref(cache.view), layer, _ptr(q), _ptr(out), _ptr(lse), _ptr(sparsity), _ptr(seq_ids), _ptr(q_pos), B, window,
        float(softmax_scale), _DT[q.dtype], _DT[out.dtype], int(max_ctx_pages), _ptr(ws), ws.numel(), _stream(stream)),
        "thinkv_decode_attention_sparsity")


def thinkv_gather_rows(src, dst, rows, stream=None):
    """contrast kernel: dst[i] = src[rows[i]] (2-D contiguous tensors of equal row size, rows int32)"""
    assert src.is_contiguous() and dst.is_contiguous() and src.dim() == 2 and dst.dim() == 2 and src.dtype == dst.dtype
    assert rows.dtype == torch.int32 and rows.is_contiguous() and dst.shape[0] == rows.numel() and dst.shape[1] == src.shape[1]
    _check(load().thinkv_gather_rows(_ptr(src), _ptr(dst), _ptr(rows), int(rows.numel()), int(src.shape[1] * src.element_size()),
                                     _stream(stream)), "thinkv_gather_rows")


def thinkv_probe_stream_pages(cache, layer, seq_ids, checksum, stream=None):
    """measurement aid: stream the pages a full-attention decode call over seq_ids reads (checksum: one int32 device word)"""
    assert seq_ids.dtype == torch.int32 and checksum.dtype == torch.int32 and checksum.numel() >= 1
    _check(load().thinkv_probe_stream_pages(C.byref(cache.view), layer, _ptr(seq_ids), int(seq_ids.numel()), _ptr(checksum), _stream(stream)),
           "thinkv_probe_stream_pages")


def thinkv_decode_attention_valu(cache, layer, q, out, lse, seq_ids, q_pos, window, softmax_scale, max_ctx_pages, stream=None):
    _decode(load().thinkv_decode_attention_valu, cache, layer, q, out, lse, seq_ids, q_pos, window, softmax_scale,
            max_ctx_pages, stream)
