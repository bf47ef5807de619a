"""Pins of the oracle's floating-point cache formats (oracle/formats.py): every code of E4M3, E2M1 and the
ternary format against tables worked out by hand from the paper's appendix "Quantization Data Formats"
(tests/golden/format_tables.json) and, for E4M3, against the library's own 8-bit float type; the encoders
against hand-made rounding cases, brute force over all codes, and the library's conversion; the group
quantisers against closed forms (exactly representable groups come back exactly, the largest element never
saturates by more than rounding, error bounds that follow from the spacing of the codes)."""
import json
import os

import numpy as np
import torch

from oracle import formats as F

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "format_tables.json")))


def test_decode_tables_match_the_hand_made_ones():
    assert np.array_equal(F.E2M1_VALUES, np.array(GOLD["e2m1_values_codes_0_to_15"]))
    assert np.array_equal(np.signbit(F.E2M1_VALUES), np.signbit(np.array(GOLD["e2m1_values_codes_0_to_15"])))
    assert np.array_equal(F.TERNARY_VALUES, np.array(GOLD["ternary_values_codes_0_to_3"]))
    for code, val in GOLD["e4m3_landmarks"].items():
        assert F.E4M3_VALUES[int(code)] == val, code
    assert np.isnan(F.E4M3_VALUES[0x7F]) and np.isnan(F.E4M3_VALUES[0xFF]) and np.isfinite(np.delete(F.E4M3_VALUES, [0x7F, 0xFF])).all()
    # structure: sign symmetry, strictly increasing magnitudes, gradual underflow (codes 0..8 equally spaced)
    assert np.array_equal(F.E4M3_VALUES[0x80:0xFF], -F.E4M3_VALUES[0x00:0x7F])
    assert (np.diff(F.E4M3_VALUES[:0x7F]) > 0).all() and np.allclose(np.diff(F.E4M3_VALUES[:9]), 2.0 ** -9, rtol=0, atol=0)


def test_e4m3_equals_the_library_type_on_every_code():
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    assert np.array_equal(np.isnan(lib), np.isnan(F.E4M3_VALUES))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], F.E4M3_VALUES[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(F.E4M3_VALUES[ok]))


def test_encoders_hand_made_rounding_cases():
    for x, want in GOLD["e2m1_rounding"]:
        assert F.e2m1_decode(F.e2m1_encode(x)) == want, x
    for x, want in GOLD["e4m3_rounding"]:
        assert F.e4m3_decode(F.e4m3_encode(x)) == want, x
    for x, want in GOLD["ternary_rounding"]:
        assert F.ternary_decode(F.ternary_encode(x)) == want, x
    assert F.e4m3_encode(np.nan) == 0x7F


def test_encoders_brute_force():
    rng = np.random.default_rng(0)
    # every representable value encodes to itself; a random value encodes to a nearest representable one (ties: even code)
    for values, enc, dec, top in ((F.E4M3_VALUES, F.e4m3_encode, F.e4m3_decode, 448.0), (F.E2M1_VALUES, F.e2m1_encode, F.e2m1_decode, 6.0)):
        finite = values[np.isfinite(values)]
        assert np.array_equal(dec(enc(finite)), finite)
        x = np.concatenate([rng.uniform(-1.2 * top, 1.2 * top, 20000), rng.normal(0, 0.05, 20000), (finite[:-1] + finite[1:]) / 2])
        got = dec(enc(x))
        best = np.abs(np.clip(x, -top, top)[:, None] - finite[None, :]).min(1)
        assert np.all(np.abs(np.clip(x, -top, top) - got) <= best + 1e-15)
        # exact midpoints go to the code with the even mantissa
        pos = finite[finite >= 0]
        pos = np.sort(pos)
        mids = (pos[:-1] + pos[1:]) / 2
        codes = enc(mids)
        assert np.all(codes % 2 == 0), "a tie went to an odd code"
    x = rng.uniform(-3, 3, 5000)
    assert np.array_equal(F.ternary_decode(F.ternary_encode(x)), np.where(np.abs(x) > 0.5, np.sign(x), 0.0))


def test_e4m3_encoder_equals_the_library_conversion_in_range():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.uniform(-448, 448, 50000), rng.normal(0, 1, 50000), rng.normal(0, 0.01, 50000)]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = F.e4m3_encode(x.astype(np.float64))
    assert np.array_equal(F.e4m3_decode(mine), F.e4m3_decode(lib))            # -0 and +0 compare equal


def test_scale_rounds_up_and_covers_the_group():
    rng = np.random.default_rng(2)
    x = rng.normal(0, 1, (200, 64)) * rng.choice([0.01, 1.0, 30.0], (200, 1))
    for quant, deq, qmax, step_rel in ((F.nvfp4_quantize, F.nvfp4_dequantize, 6.0, 1.0), (F.ternary_quantize, F.ternary_dequantize, 1.0, 0.5)):
        codes, sc = quant(x)
        s = F.e4m3_decode(sc)
        amax = np.abs(x.reshape(200, 4, 16)).max(-1)
        assert np.all(s * qmax >= amax) and np.all(F.e4m3_decode(np.maximum(sc.astype(int) - 1, 0)) * qmax < amax + 1e-300)
        err = np.abs(deq(codes, sc) - x).reshape(200, 4, 16)
        # nothing saturates, so the error is at most half the widest gap between neighbouring codes, times the scale
        assert np.all(err <= s[..., None] * step_rel + 1e-12)
    # a group of zeros: scale 0, codes 0, decodes to zeros; a group on the grid comes back exactly
    c, sc = F.nvfp4_quantize(np.zeros((1, 16)))
    assert not c.any() and not sc.any() and not F.nvfp4_dequantize(c, sc).any()
    grid = np.array([[0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.5, -1, -1.5, -2, -3, -4, -6, 0]]) * 0.25     # scale 0.25 is an E4M3 value
    c, sc = F.nvfp4_quantize(grid)
    assert np.array_equal(F.nvfp4_dequantize(c, sc), grid) and F.e4m3_decode(sc)[0, 0] == 0.25
    tern = np.array([[2.0, -2.0, 0, 0, 2.0, 0, -2.0, 0, 0, 0, 0, 0, 0, 0, 0, 2.0]])
    c, sc = F.ternary_quantize(tern)
    assert np.array_equal(F.ternary_dequantize(c, sc), tern) and set(np.unique(c)) <= {0, 1, 3}
    # FP8 with a per-tensor scale: relative error at most 2^-4 for values in the normal range
    y = rng.normal(0, 2, 1000)
    back = F.fp8_dequantize(F.fp8_quantize(y, 0.05), 0.05)
    big = np.abs(y) > 0.05 * 2.0 ** -6
    assert np.all(np.abs(back[big] - y[big]) <= np.abs(y[big]) * 2.0 ** -4)


# ------------------------------------------------- the formats inside the paged cache (layout, bookkeeping, attention)
def _read_fp_block_bit_by_bit(img, bits, D):
    """independent reader of a (page, kv-head) block in the paper's formats: code regions as for the integer formats
    (the chunk formulas at the top of oracle/layout.py), one scale byte per (slot, group of 16) at group16*16 + slot"""
    from oracle import layout
    cb = layout.chunk_bytes(bits, D)
    meta = 0 if bits == 8 else 16 * (D // 16)
    offs = (0, 64 * cb, 64 * cb + meta, 2 * 64 * cb + meta)
    fph = 16 // bits
    kc = np.zeros((16, D), np.uint8)
    vc = np.zeros((16, D), np.uint8)
    for lane in range(64):
        kchunk = int.from_bytes(img[offs[0] + lane * cb: offs[0] + (lane + 1) * cb].tobytes(), "little")
        vchunk = int.from_bytes(img[offs[2] + lane * cb: offs[2] + (lane + 1) * cb].tobytes(), "little")
        for f in range(cb * 8 // bits // 2):
            for h in range(2):
                off = 32 * (f // fph) + 16 * h + bits * (f % fph)
                j, t = lane // 16, lane % 16
                kc[t, 32 * (f // 4) + 8 * j + 2 * (f % 4) + h] = (kchunk >> off) & ((1 << bits) - 1)
                q, m = lane // 16, lane % 16
                u, mb = f // (D // 16), f % (D // 16)
                vc[4 * q + 2 * u + h, 16 * mb + m] = (vchunk >> off) & ((1 << bits) - 1)
    ks = vs = None
    if bits != 8:
        ks = np.array([[img[offs[1] + g * 16 + t] for g in range(D // 16)] for t in range(16)], np.uint8)
        vs = np.array([[img[offs[3] + g * 16 + t] for g in range(D // 16)] for t in range(16)], np.uint8)
    return kc, ks, vc, vs


def test_fp_block_layout_round_trips_through_an_independent_reader():
    from oracle import layout
    for D in (64, 128):
        for bits in (2, 4, 8):
            rng = np.random.default_rng(bits * D + 1)
            kc = rng.integers(0, 1 << bits, (16, D), dtype=np.uint8)
            vc = rng.integers(0, 1 << bits, (16, D), dtype=np.uint8)
            ks = rng.integers(0, 127, (16, D // 16), dtype=np.uint8)
            vs = rng.integers(0, 127, (16, D // 16), dtype=np.uint8)
            img = layout.pack_page_head_fp(kc, ks, vc, vs, bits)
            assert img.size == layout.block_bytes_fp(bits, D) == 16 * 2 * (D * bits // 8 + (0 if bits == 8 else D // 16))
            gk, gks, gv, gvs = _read_fp_block_bit_by_bit(img, bits, D)
            assert np.array_equal(gk, kc) and np.array_equal(gv, vc)
            if bits != 8:
                assert np.array_equal(gks, ks) and np.array_equal(gvs, vs)


def test_cache_in_the_papers_formats():
    """the paged cache with fmt='fp': what it stores is the formats' quantiser output, what attention sees is its decode,
    and attention over it equals dense softmax attention over those decoded tokens (evicted == absent)"""
    from oracle import attention, cache as oc
    cfg = oc.OracleConfig(1, 8, 2, 64, (2, 4, 8), 1, 16, (16, 16, 16), fmt="fp", fp8_scale=(0.04, 0.06))     # the paper's map: T2 / E4 / R8
    c = oc.OracleCache(cfg)
    rng = np.random.default_rng(3)
    n = 90
    k = rng.standard_normal((n, 2, 64)).astype(np.float16).astype(np.float32)
    v = rng.standard_normal((n, 2, 64)).astype(np.float16).astype(np.float32)
    v[:, :, 5] *= 8
    cls = rng.integers(0, 3, n).astype(np.uint8)
    h = c.append(0, k, v, np.zeros(n, np.int64), np.arange(n), cls)
    assert (h >= 0).all()
    c.evict_slots(0, [0] * 10, h[20:30])
    # stored codes and scales are the formats' own
    for i in (0, 7, 50, 89):
        cc, pi, slot = oc.split_handle(h[i])
        pid = int(c.table[0, 0, cc, pi])
        bits = cfg.bits_of_class[cc]
        if bits == 8:
            want = F.fp8_quantize(v[i], 0.06)
        else:
            want, sc = (F.nvfp4_quantize if bits == 4 else F.ternary_quantize)(v[i])
            assert np.array_equal(c.v_scale[cc][pid, :, slot, :], sc)
        assert np.array_equal(c.v_codes[cc][pid, :, slot, :], want)
    q = rng.standard_normal((1, 8, 64))
    out, lse = attention.decode_attention(c, 0, q, [0], [n - 1], 0, 0.125)
    keep = np.r_[0:20, 30:n]
    kd = np.zeros((len(keep), 2, 64))
    vd = np.zeros((len(keep), 2, 64))
    for r, i in enumerate(keep):
        bits = cfg.bits_of_class[cls[i]]
        for src, dst, ts in ((k, kd, 0.04), (v, vd, 0.06)):
            if bits == 8:
                dst[r] = F.fp8_dequantize(F.fp8_quantize(src[i], ts), ts)
            elif bits == 4:
                dst[r] = F.nvfp4_dequantize(*F.nvfp4_quantize(src[i]))
            else:
                dst[r] = F.ternary_dequantize(*F.ternary_quantize(src[i]))
    for hq in range(8):
        sc = 0.125 * kd[:, hq // 4, :] @ q[0, hq]
        p = np.exp(sc - sc.max())
        assert np.allclose(out[0, hq], (p / p.sum()) @ vd[:, hq // 4, :], rtol=1e-12, atol=1e-12)
    # bytes: 2-bit 2*(16+4), 4-bit 2*(32+4), 8-bit 2*64 per token and kv-head at D = 64
    assert [c.token_bytes(t) for t in range(3)] == [40, 72, 128]
    img = c.arena_image(1)
    assert img.shape[1] == 2 * 16 * 72
