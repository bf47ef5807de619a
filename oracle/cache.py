"""Paged KV cache bookkeeping model (test infrastructure; see oracle/__init__.py).

A sequential, one-token-at-a-time statement of the paper's Continuous Thinking memory
manager (Sec. 5.2 "Continuous Thinking (CT)" and the appendix "ThinKV Walkthrough Example"):

  * one block table per request and per layer; every block holds tokens of ONE thought type
    (thought-aware paging) -- kept here as one page list per (request, layer, type), which is
    the paper's table sorted by its "thought type" column;
  * eviction only sets a bit in the block's eviction mask; no data moves ("TBE with CT");
  * a new token of type c goes to a reclaimable (evict-marked) slot of an existing block of
    type c and clears that mask bit; otherwise to the next never-used slot of the last block of
    type c; otherwise to a newly allocated block -- never to a block of another type
    ("Efficient Memory Management", walkthrough steps a-d).

Readings where the paper is silent (each also listed in the design notes):
  * among several reclaimable slots: first page in table order, lowest slot index;
  * the per-type free pool hands out physical pages 0,1,2,... (a LIFO stack seeded that way);
  * a fully evicted block stays owned by its (request, layer, type);
  * evicting a slot that holds no live token is an ignored, flagged no-op;
  * attention never sees a slot whose live bit is clear (evicted == masked == absent).

Thought types are numbered as in the paper's pseudocode: 0 = transition (T), 1 = execution
(E), 2 = reasoning (R).  The bit width of each type is a parameter (bits_of_class).
"""
from dataclasses import dataclass, field
import numpy as np

from . import formats, layout, quant

PAGE = layout.PAGE
ST_NOPAGES, ST_BAD_CLASS, ST_BAD_SLOT, ST_EVICT_DEAD, ST_BAD_SEQ = 1, 2, 4, 8, 16


def make_handle(c, page_idx, slot):
    return (c << 28) | (page_idx << 4) | slot


def split_handle(h):
    h = int(h) & 0xFFFFFFFF
    return h >> 28, (h >> 4) & 0xFFFFFF, h & 15


@dataclass
class OracleConfig:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    bits_of_class: tuple            # index 0=T, 1=E, 2=R
    max_seqs: int
    max_pages: int                  # per (sequence, layer, class) page list
    arena_pages: tuple              # physical pages per class
    page_size: int = PAGE
    group_size: int = quant.GROUP
    fmt: str = "int"                # "int": asymmetric integer codes, binary16 scale and zero-point per 32 (quant.py);
                                    # "fp": the paper's formats (formats.py): 8 bits = E4M3 with one scale per tensor,
                                    # 4 bits = E2M1 and 2 bits = ternary with an E4M3 scale per 16 channels of the token
    fp8_scale: tuple = (1.0, 1.0)   # fmt "fp": the per-tensor binary32 scales of keys and of values (from calibration)


class OracleCache:
    def __init__(self, cfg: OracleConfig, store_data=True):
        assert cfg.page_size == PAGE and cfg.group_size == quant.GROUP and cfg.fmt in ("int", "fp")
        self.cfg = cfg
        self.store_data = store_data
        S, L, MP = cfg.max_seqs, cfg.n_layers, cfg.max_pages
        H, D, NG = cfg.n_kv_heads, cfg.head_dim, cfg.head_dim // quant.GROUP
        self.table = np.full((S, L, 3, MP), -1, dtype=np.int32)
        self.n_pages = np.zeros((S, L, 3), dtype=np.int32)
        self.n_live = np.zeros((S, L), dtype=np.int32)
        self.status = np.zeros(S * L + 1, dtype=np.uint32)
        self.free_stack, self.free_top = [], np.zeros(3, dtype=np.int32)
        self.filled, self.valid, self.evict, self.slot_pos = [], [], [], []
        self.k_codes, self.v_codes, self.k_scale, self.k_zp, self.v_scale, self.v_zp = [], [], [], [], [], []
        for c in range(3):
            n = int(cfg.arena_pages[c])
            self.free_stack.append(np.arange(n - 1, -1, -1, dtype=np.int32))   # top of stack = page 0
            self.free_top[c] = n
            self.filled.append(np.zeros(n, dtype=np.uint8))
            self.valid.append(np.zeros(n, dtype=np.uint16))
            self.evict.append(np.zeros(n, dtype=np.uint16))
            self.slot_pos.append(np.full((n, PAGE), -1, dtype=np.int32))
            nd = n if store_data else 0
            self.k_codes.append(np.zeros((nd, H, PAGE, D), dtype=np.uint8))
            self.v_codes.append(np.zeros((nd, H, PAGE, D), dtype=np.uint8))
            if cfg.fmt == "int":
                for lst in (self.k_scale, self.k_zp, self.v_scale, self.v_zp):
                    lst.append(np.zeros((nd, H, PAGE, NG), dtype=np.float16))
            else:   # E4M3 scale codes per 16 channels (unused by the 8-bit type); no zero-points
                for lst in (self.k_scale, self.v_scale):
                    lst.append(np.zeros((nd, H, PAGE, D // formats.GROUP16), dtype=np.uint8))
                for lst in (self.k_zp, self.v_zp):
                    lst.append(None)

    # ------------------------------------------------------------------ append
    def _select_slot(self, s, l, c):
        """Returns (page_idx, slot) or None when no page can be had."""
        cfg = self.cfg
        n = int(self.n_pages[s, l, c])
        pages = self.table[s, l, c, :n]
        ev = self.evict[c][pages]
        hit = np.flatnonzero(ev)
        if hit.size:                                     # reclaim an evicted slot in place
            pi = int(hit[0])
            m = int(ev[pi])
            return pi, (m & -m).bit_length() - 1
        if n and self.filled[c][pages[-1]] < PAGE:       # next never-used slot of the last block
            return n - 1, int(self.filled[c][pages[-1]])
        if n == cfg.max_pages or self.free_top[c] == 0:
            return None
        self.free_top[c] -= 1
        pid = int(self.free_stack[c][self.free_top[c]])
        self.filled[c][pid] = 0
        self.valid[c][pid] = 0
        self.evict[c][pid] = 0
        self.slot_pos[c][pid, :] = -1
        self.table[s, l, c, n] = pid
        self.n_pages[s, l, c] = n + 1
        return n, 0

    def append(self, layer, k_new, v_new, tok_seq, tok_pos, tok_class):
        """k_new, v_new: [n_tok, Hkv, D] (values exactly representable in binary32).
        Tokens are applied in array order.  Returns int32 handles [n_tok] (-1 = skipped)."""
        cfg = self.cfg
        if self.store_data:
            k_new = np.asarray(k_new, dtype=np.float32)
            v_new = np.asarray(v_new, dtype=np.float32)
        tok_class = np.asarray(tok_class)
        n_tok = len(tok_seq)
        handles = np.full(n_tok, -1, dtype=np.int32)
        q = {}
        if self.store_data:
            for c in range(3):
                idx = np.flatnonzero(tok_class == c)
                if idx.size:
                    b = cfg.bits_of_class[c]
                    q[c] = (dict(zip(idx.tolist(), range(idx.size))), self._quantize(k_new[idx], b, 0), self._quantize(v_new[idx], b, 1))
        for i in range(n_tok):
            s, pos, c = int(tok_seq[i]), int(tok_pos[i]), int(tok_class[i])
            if not 0 <= s < cfg.max_seqs:
                self.status[-1] |= ST_BAD_SEQ
                continue
            sl = s * cfg.n_layers + layer
            if not 0 <= c <= 2:
                self.status[sl] |= ST_BAD_CLASS
                continue
            sel = self._select_slot(s, layer, c)
            if sel is None:
                self.status[sl] |= ST_NOPAGES
                continue
            pi, slot = sel
            pid = int(self.table[s, layer, c, pi])
            bit = np.uint16(1 << slot)
            if slot >= self.filled[c][pid]:
                assert slot == self.filled[c][pid]
                self.filled[c][pid] = slot + 1
            self.evict[c][pid] &= ~bit
            self.valid[c][pid] |= bit
            self.slot_pos[c][pid, slot] = pos
            self.n_live[s, layer] += 1
            if self.store_data:
                row, (kc, ks, kz), (vc, vs, vz) = q[c][0][i], q[c][1], q[c][2]
                self.k_codes[c][pid, :, slot, :] = kc[row]
                self.v_codes[c][pid, :, slot, :] = vc[row]
                if ks is not None:
                    self.k_scale[c][pid, :, slot, :] = ks[row]
                    self.v_scale[c][pid, :, slot, :] = vs[row]
                if kz is not None:
                    self.k_zp[c][pid, :, slot, :] = kz[row]
                    self.v_zp[c][pid, :, slot, :] = vz[row]
            handles[i] = make_handle(c, pi, slot)
        return handles

    # --------------------------------------------------------- number formats
    def _quantize(self, x, bits, kind):
        """(codes, scales or None, zero-points or None) of rows x [n, Hkv, D]; kind 0 = keys, 1 = values"""
        if self.cfg.fmt == "int":
            return quant.quantize_groups(x, bits)
        if bits == 8:
            return formats.fp8_quantize(x, self.cfg.fp8_scale[kind]), None, None
        codes, sc = (formats.nvfp4_quantize if bits == 4 else formats.ternary_quantize)(x)
        return codes, sc, None

    def dequant(self, c, kind, pids, slots):
        """binary64 values [n, Hkv, D] of the listed (page, slot) pairs of class c; kind 0 = keys, 1 = values"""
        codes = (self.v_codes if kind else self.k_codes)[c][pids, :, slots, :]
        scale = (self.v_scale if kind else self.k_scale)[c][pids, :, slots, :]
        if self.cfg.fmt == "int":
            zp = (self.v_zp if kind else self.k_zp)[c][pids, :, slots, :]
            return quant.dequantize(codes, scale, zp)
        bits = self.cfg.bits_of_class[c]
        if bits == 8:
            return formats.fp8_dequantize(codes, self.cfg.fp8_scale[kind])
        return (formats.nvfp4_dequantize if bits == 4 else formats.ternary_dequantize)(codes, scale)

    def token_bytes(self, c):
        """K + V bytes one token of class c occupies per kv-head"""
        b, D = self.cfg.bits_of_class[c], self.cfg.head_dim
        if self.cfg.fmt == "int":
            return 2 * (D * b // 8 + D // quant.GROUP * 4)
        return 2 * (D * b // 8 + (0 if b == 8 else D // formats.GROUP16))

    # ------------------------------------------------------------------- evict
    def evict_slots(self, layer, ev_seq, ev_handle):
        cfg = self.cfg
        for s, h in zip(ev_seq, ev_handle):
            s = int(s)
            if not 0 <= s < cfg.max_seqs:
                self.status[-1] |= ST_BAD_SEQ
                continue
            sl = s * cfg.n_layers + layer
            if int(h) == -1:
                continue                           # placeholder: no token
            c, pi, slot = split_handle(h)
            if int(h) < 0 or c > 2 or pi >= self.n_pages[s, layer, c]:
                self.status[sl] |= ST_BAD_SLOT
                continue
            pid = int(self.table[s, layer, c, pi])
            bit = np.uint16(1 << slot)
            if self.valid[c][pid] & bit:
                self.valid[c][pid] &= ~bit
                self.evict[c][pid] |= bit          # soft mark; the slot's bytes stay as they are
                self.n_live[s, layer] -= 1
            else:
                self.status[sl] |= ST_EVICT_DEAD

    # ---------------------------------------------------------------- queries
    def live_tokens(self, s, layer):
        """[(pos, class, page_id, slot)] of every live token, in table order."""
        out = []
        for c in range(3):
            for pi in range(int(self.n_pages[s, layer, c])):
                pid = int(self.table[s, layer, c, pi])
                m = int(self.valid[c][pid])
                for slot in range(PAGE):
                    if m >> slot & 1:
                        out.append((int(self.slot_pos[c][pid, slot]), c, pid, slot))
        return out

    def arena_image(self, c, n_pages=None):
        """uint8 [n_pages, page_bytes] image of the first n_pages physical pages of class c."""
        n = self.k_codes[c].shape[0] if n_pages is None else n_pages
        return self.arena_image_pages(c, np.arange(n))

    def arena_image_pages(self, c, pids):
        """uint8 [len(pids), page_bytes] image of the listed physical pages of class c"""
        b = self.cfg.bits_of_class[c]
        p = np.asarray(pids, dtype=np.int64)
        if self.cfg.fmt == "int":
            img = layout.pack_page_head(self.k_codes[c][p], self.k_scale[c][p], self.k_zp[c][p],
                                        self.v_codes[c][p], self.v_scale[c][p], self.v_zp[c][p], b)
        else:
            img = layout.pack_page_head_fp(self.k_codes[c][p], self.k_scale[c][p], self.v_codes[c][p], self.v_scale[c][p], b)
        return img.reshape(len(p), -1)

    def stored_bytes_live(self, s, layer):
        """K+V bytes the live tokens of (s, layer) occupy: per token and kv-head
        2*(D*b/8 + (D/32)*4)  (codes plus a binary16 scale and zero-point per group)."""
        cfg = self.cfg
        tot = 0
        for _, c, _, _ in self.live_tokens(s, layer):
            tot += cfg.n_kv_heads * self.token_bytes(c)
        return tot
