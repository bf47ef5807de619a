"""Pins for the oracle's paged-cache bookkeeping (CPU only)."""
import numpy as np
import pytest

from oracle import cache as oc
from oracle import quant

R, E, T = 2, 1, 0


def _cfg(bits=(8, 2, 4), max_pages=8, arena=(8, 8, 8), layers=1, seqs=2, D=64, H=2):
    return oc.OracleConfig(layers, 4 * H, H, D, bits, seqs, max_pages, arena)


def _rows(n, H=2, D=64, seed=0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, H, D)).astype(np.float16).astype(np.float32),
            rng.standard_normal((n, H, D)).astype(np.float16).astype(np.float32))


def _append(c, cls, pos0, n, seq=0, layer=0, seed=0):
    k, v = _rows(n, c.cfg.n_kv_heads, c.cfg.head_dim, seed)
    return c.append(layer, k, v, np.full(n, seq), np.arange(pos0, pos0 + n), np.full(n, cls))


def test_walkthrough_events():
    """The events of the paper's appendix 'ThinKV Walkthrough Example' (steps a-d), at this
    build's block size of 16.  The figure with the exact slot numbers is not available, so the
    events are tested, not the slot numbers."""
    c = oc.OracleCache(_cfg())
    # step a: first reasoning tokens -> a new table entry of type 2, a physical block, masks clear
    h = _append(c, R, 0, 16)
    assert c.n_pages[0, 0].tolist() == [0, 0, 1]
    pidR = c.table[0, 0, R, 0]
    assert c.evict[R][pidR] == 0 and c.valid[R][pidR] == 0xFFFF and c.filled[R][pidR] == 16
    # step b: execution tokens get their own block even while ... (here R is full; make room first)
    c2 = oc.OracleCache(_cfg())
    _append(c2, R, 0, 5)
    _append(c2, E, 5, 4)
    assert c2.n_pages[0, 0].tolist() == [0, 1, 1]          # not placed in the half-empty R block
    assert c2.filled[R][c2.table[0, 0, R, 0]] == 5 and c2.filled[E][c2.table[0, 0, E, 0]] == 4
    # step c: transition tokens, then eviction only flips mask bits -- no byte of data moves
    _append(c, E, 16, 4)
    _append(c, T, 20, 4)
    before = [c.arena_image(k).copy() for k in range(3)]
    c.evict_slots(0, [0, 0], [h[3], h[9]])
    assert c.evict[R][pidR] == (1 << 3) | (1 << 9)
    assert c.valid[R][pidR] == 0xFFFF & ~((1 << 3) | (1 << 9))
    assert all(np.array_equal(a, c.arena_image(k)) for k, a in enumerate(before))
    assert c.n_live[0, 0] == 22
    # step d: two reasoning tokens land in the two freed slots of that block; mask back to all 0
    h2 = _append(c, R, 24, 2, seed=5)
    assert [oc.split_handle(x) for x in h2] == [(R, 0, 3), (R, 0, 9)]
    assert c.evict[R][pidR] == 0 and c.valid[R][pidR] == 0xFFFF
    assert c.slot_pos[R][pidR, 3] == 24 and c.slot_pos[R][pidR, 9] == 25
    # ... the next two find no empty slot: a new block is allocated
    h3 = _append(c, R, 26, 2, seed=6)
    assert [oc.split_handle(x) for x in h3] == [(R, 1, 0), (R, 1, 1)]
    assert c.n_pages[0, 0, R] == 2 and c.n_live[0, 0] == 26


def test_same_width_classes_never_share_a_block():
    c = oc.OracleCache(_cfg(bits=(2, 4, 4)))           # the paper's practical R4E4T2 map
    _append(c, R, 0, 3)
    _append(c, E, 3, 3)
    assert c.n_pages[0, 0].tolist() == [0, 1, 1]


def test_page_ids_come_out_in_order_and_pool_exhaustion_is_flagged():
    c = oc.OracleCache(_cfg(arena=(2, 2, 2), max_pages=4))
    h = _append(c, T, 0, 40)                               # needs 3 pages, pool has 2
    assert c.table[0, 0, T, :2].tolist() == [0, 1]
    assert (h[:32] >= 0).all() and (h[32:] == -1).all()
    assert c.status[0] & oc.ST_NOPAGES and c.n_live[0, 0] == 32
    h = _append(c, E, 40, 1, seq=1)
    assert c.table[1, 0, E, 0] == 0 and c.status[1] == 0


def test_flagged_noops():
    c = oc.OracleCache(_cfg())
    h = _append(c, R, 0, 4)
    c.evict_slots(0, [0], [h[1]])
    c.evict_slots(0, [0], [h[1]])                          # already evicted
    assert c.status[0] == oc.ST_EVICT_DEAD and c.n_live[0, 0] == 3
    c.evict_slots(0, [0], [oc.make_handle(R, 0, 9)])       # never filled
    assert c.n_live[0, 0] == 3
    c.status[:] = 0
    c.evict_slots(0, [0], [oc.make_handle(E, 0, 0)])       # no such page
    assert c.status[0] == oc.ST_BAD_SLOT
    k, v = _rows(1)
    assert c.append(0, k, v, [0], [9], [3])[0] == -1 and c.status[0] & oc.ST_BAD_CLASS
    assert c.append(0, k, v, [7], [9], [1])[0] == -1 and c.status[-1] & oc.ST_BAD_SEQ


class DictModel:
    """A second, deliberately different model: every (seq, layer, class) is a plain list of
    pages, each a list of 16 cells that are None (never used), ('live', pos) or ('dead', pos);
    the placement rule is re-derived from the paper's prose by scanning cells one by one."""

    def __init__(self):
        self.pages = {}

    def append(self, key, pos):
        pages = self.pages.setdefault(key, [])
        for pi, pg in enumerate(pages):                      # a reclaimable cell anywhere, first found
            for si, cell in enumerate(pg):
                if cell is not None and cell[0] == 'dead':
                    pg[si] = ('live', pos)
                    return pi, si
        if pages:
            pg = pages[-1]
            for si, cell in enumerate(pg):
                if cell is None:
                    pg[si] = ('live', pos)
                    return len(pages) - 1, si
        pages.append([None] * 16)
        pages[-1][0] = ('live', pos)
        return len(pages) - 1, 0

    def evict(self, key, pi, si):
        cell = self.pages[key][pi][si]
        if cell is not None and cell[0] == 'live':
            self.pages[key][pi][si] = ('dead', cell[1])


def check_invariants(c):
    cfg = c.cfg
    seen = [set(), set(), set()]
    live = np.zeros_like(c.n_live)
    for s in range(cfg.max_seqs):
        for l in range(cfg.n_layers):
            poss = []
            for k in range(3):
                for pi in range(c.n_pages[s, l, k]):
                    pid = int(c.table[s, l, k, pi])
                    assert pid not in seen[k]
                    seen[k].add(pid)
                    v, e, f = int(c.valid[k][pid]), int(c.evict[k][pid]), int(c.filled[k][pid])
                    assert v & e == 0
                    assert bin(v).count("1") + bin(e).count("1") == f
                    assert (v | e) == (1 << f) - 1
                    live[s, l] += bin(v).count("1")
                    poss += [int(c.slot_pos[k][pid, i]) for i in range(16) if v >> i & 1]
            assert len(poss) == len(set(poss))
    assert np.array_equal(live, c.n_live)
    for k in range(3):
        free = set(c.free_stack[k][:c.free_top[k]].tolist())
        assert free.isdisjoint(seen[k]) and len(free) + len(seen[k]) == cfg.arena_pages[k]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_ops_against_the_dict_model(seed):
    rng = np.random.default_rng(seed)
    cfg = _cfg(max_pages=64, arena=(96, 96, 96), layers=2, seqs=3)
    c = oc.OracleCache(cfg, store_data=False)
    m = DictModel()
    handle_of = {}
    nxt = np.zeros((3, 2), dtype=int)
    for step in range(300):
        l = int(rng.integers(2))
        if rng.random() < 0.7 or not handle_of:
            n = int(rng.integers(1, 24))
            seqs = np.sort(rng.integers(0, 3, n))
            cls = rng.integers(0, 3, n)
            pos = np.zeros(n, dtype=int)
            for i, s in enumerate(seqs):
                pos[i] = nxt[s, l]
                nxt[s, l] += 1
            z = np.zeros((n, 2, 64), dtype=np.float32)
            h = c.append(l, z, z, seqs, pos, cls)
            for i in range(n):
                want = m.append((int(seqs[i]), l, int(cls[i])), int(pos[i]))
                assert oc.split_handle(h[i]) == (int(cls[i]), want[0], want[1])
                handle_of[(int(seqs[i]), l, int(pos[i]))] = int(h[i])
        else:
            keys = [k for k in handle_of if k[1] == l]
            if not keys:
                continue
            pick = [keys[i] for i in rng.choice(len(keys), size=min(len(keys), int(rng.integers(1, 40))), replace=False)]
            c.evict_slots(l, [k[0] for k in pick], [handle_of[k] for k in pick])
            for k in pick:
                cc, pi, si = oc.split_handle(handle_of[k])
                m.evict((k[0], l, cc), pi, si)
                del handle_of[k]
        if step % 25 == 0:
            check_invariants(c)
    check_invariants(c)
    # final state agrees cell by cell
    for (s, l, k), pages in m.pages.items():
        assert c.n_pages[s, l, k] == len(pages)
        for pi, pg in enumerate(pages):
            pid = int(c.table[s, l, k, pi])
            for si, cell in enumerate(pg):
                assert bool(c.valid[k][pid] >> si & 1) == (cell is not None and cell[0] == 'live')
                assert bool(c.evict[k][pid] >> si & 1) == (cell is not None and cell[0] == 'dead')
                if cell is not None:
                    assert c.slot_pos[k][pid, si] == cell[1]


def test_byte_accounting_matches_the_memory_model():
    """Sec. 3 'Memory footprint': bytes grow as (tokens kept) x (average bits).  With three
    classes the stored K+V bytes are sum over live tokens of 2*Hkv*(D*b/8 + (D/32)*4)."""
    cfg = _cfg(bits=(8, 2, 4))
    c = oc.OracleCache(cfg)
    hT = _append(c, T, 0, 10)
    hE = _append(c, E, 10, 20)
    hR = _append(c, R, 30, 7)
    c.evict_slots(0, [0] * 5, hE[:5])
    per = lambda b: 2 * 2 * (64 * b // 8 + 2 * 4)
    assert c.stored_bytes_live(0, 0) == 10 * per(8) + 15 * per(2) + 7 * per(4)
    assert per(8) == 2 * 144 and per(4) == 2 * 80 and per(2) == 2 * 48


def test_stored_codes_are_the_reference_quantiser_output():
    cfg = _cfg()
    c = oc.OracleCache(cfg)
    k, v = _rows(3)
    h = c.append(0, k, v, [0, 0, 0], [0, 1, 2], [E, R, E])
    cc, pi, si = oc.split_handle(h[2])
    pid = c.table[0, 0, cc, pi]
    codes, s, z = quant.quantize_groups(v[2], cfg.bits_of_class[E])
    assert np.array_equal(c.v_codes[E][pid, :, si, :], codes)
    assert np.array_equal(c.v_scale[E][pid, :, si, :].view(np.uint16), s.view(np.uint16))
