"""Pins for the reference quantizer and the page byte layout (CPU only)."""
import json
import os

import numpy as np
import pytest

from oracle import layout, quant

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _draw(rng, n, dtype):
    import torch
    x = torch.from_numpy(rng.standard_normal((n, 128)).astype(np.float32))
    x[:, [3, 17, 69, 126]] *= 8
    return x.to(dtype).float().numpy()


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_round_trip_error_at_most_half_a_step(bits, dt):
    import torch
    rng = np.random.default_rng(bits)
    x = _draw(rng, 512, torch.float16 if dt == "f16" else torch.bfloat16)
    c, s, z = quant.quantize_groups(x, bits)
    xh = quant.dequantize(c, s, z)
    step = np.repeat(s.astype(np.float64), 32, axis=-1)
    # zero-point is the exact group minimum for 16-bit inputs, so the bound is step/2 alone
    assert np.array_equal(z.astype(np.float32), x.reshape(512, 4, 32).min(-1))
    assert np.all(np.abs(x.astype(np.float64) - xh) <= step / 2 * (1 + 1e-12))
    assert c.max() <= (1 << bits) - 1


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_extremes_constant_and_monotone(bits):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((64, 32)).astype(np.float16).astype(np.float32)
    c, s, z = quant.quantize_groups(x, bits)
    assert np.all(c[np.arange(64), x.argmin(1)] == 0)
    assert np.all(c[np.arange(64), x.argmax(1)] == (1 << bits) - 1)
    order = np.argsort(x, axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(c.astype(int), order, 1), axis=1) >= 0)
    const = np.full((1, 32), 0.3125, dtype=np.float32)
    c, s, z = quant.quantize_groups(const, bits)
    assert s.view(np.uint16)[0, 0] == 0 and not c.any()
    assert quant.dequantize(c, s, z)[0, 0] == 0.3125


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_scale_is_the_smallest_binary16_covering_the_range(bits):
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((4096, 32)) * rng.uniform(1e-3, 30, (4096, 1))).astype(np.float16).astype(np.float32)
    _, s, _ = quant.quantize_groups(x, bits)
    rng_ = (x.max(1) - x.min(1)).astype(np.float64)
    q = (1 << bits) - 1
    s32 = ((x.max(1) - x.min(1)) / np.float32(q)).astype(np.float32)
    sf = s[:, 0].astype(np.float64)
    assert np.all(sf >= s32)                                    # never below the exact step
    below = (s[:, 0].view(np.uint16) - 1).view(np.float16).astype(np.float64)
    assert np.all(below < s32)                                  # and the next lower binary16 is
    assert np.all(q * sf >= rng_ * (1 - 2 ** -23))


def test_hand_worked_cases():
    """tests/golden/quant_cases.json: groups worked out by hand from the definition in the
    paper's appendix 'Group Quantization' under the asymmetric reading (see the file)."""
    with open(os.path.join(GOLD, "quant_cases.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        x = np.resize(np.array(case["x"], dtype=np.float32), 32)[None]
        c, s, z = quant.quantize_groups(x, case["bits"])
        n = len(case["x"])
        assert c[0, :n].tolist() == case["codes"], case["name"]
        assert float(s[0, 0]) == case["scale"], case["name"]
        assert float(z[0, 0]) == case["zp"], case["name"]


def test_negative_zero_minimum_is_canonical():
    x = np.zeros((1, 32), dtype=np.float32)
    x[0, 0] = -0.0
    x[0, 5] = 1.0
    _, _, z = quant.quantize_groups(x, 4)
    assert z.view(np.uint16)[0, 0] == 0


def test_binary32_input_below_zero_point_clamps():
    x = np.linspace(0, 1, 32, dtype=np.float32)[None].copy()
    x[0, 0] = np.float32(-1.0003)                 # binary16 zero-point becomes -1.0, above the minimum
    c, s, z = quant.quantize_groups(x, 8)
    assert c.min() == 0 and c.max() == 255


# ------------------------------------------------------------------------- layout
def _unpack_bit_by_bit(img, bits, D):
    """independent reader: walks the byte image as one big little-endian integer per chunk"""
    cb = layout.chunk_bytes(bits, D)
    ok, km_, vo, vm_ = layout.region_offsets(bits, D)
    kc = np.zeros((16, D), dtype=np.uint8)
    vc = np.zeros((16, D), dtype=np.uint8)
    fph = 16 // bits
    for lane in range(64):
        kchunk = int.from_bytes(img[ok + lane * cb: ok + (lane + 1) * cb].tobytes(), "little")
        vchunk = int.from_bytes(img[vo + lane * cb: vo + (lane + 1) * cb].tobytes(), "little")
        for f in range(cb * 8 // bits // 2):
            for h in range(2):
                off = 32 * (f // fph) + 16 * h + bits * (f % fph)
                kcode = (kchunk >> off) & ((1 << bits) - 1)
                vcode = (vchunk >> off) & ((1 << bits) - 1)
                # K chunk lane = 16*j + t holds channels 32*g + 8*j + e, e = 2*(f%4)+h, g = f//4
                j, t = lane // 16, lane % 16
                kc[t, 32 * (f // 4) + 8 * j + 2 * (f % 4) + h] = kcode
                # V chunk lane = 16*q + m holds slots 4q + 2u + h, channels 16*mb + m, f = u*(D/16)+mb
                q, m = lane // 16, lane % 16
                u, mb = f // (D // 16), f % (D // 16)
                vc[4 * q + 2 * u + h, 16 * mb + m] = vcode
    ng = D // 32
    def meta(o):
        """binary16 number i of a meta region: unit i//8 = group*4 + slot quad; i%8 < 4 scale, else zero-point"""
        sc = np.zeros((16, ng), dtype=np.float16)
        zp = np.zeros((16, ng), dtype=np.float16)
        for i in range(16 * ng * 2):
            val = np.array([int.from_bytes(img[o + 2 * i:o + 2 * i + 2].tobytes(), "little")], dtype=np.uint16).view(np.float16)[0]
            unit, e = divmod(i, 8)
            grp, quad = divmod(unit, 4)
            (sc if e < 4 else zp)[4 * quad + e % 4, grp] = val
        return sc, zp
    ks, kz = meta(km_)
    vs, vz = meta(vm_)
    return kc, ks, kz, vc, vs, vz


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_pack_round_trips_through_an_independent_reader(bits, D):
    rng = np.random.default_rng(bits * D)
    kc = rng.integers(0, 1 << bits, (16, D), dtype=np.uint8)
    vc = rng.integers(0, 1 << bits, (16, D), dtype=np.uint8)
    m = [rng.standard_normal((16, D // 32)).astype(np.float16) for _ in range(4)]
    img = layout.pack_page_head(kc, m[0], m[1], vc, m[2], m[3], bits)
    assert img.size == layout.block_bytes(bits, D) == 16 * 2 * (D * bits // 8 + D // 32 * 4)
    got = _unpack_bit_by_bit(img, bits, D)
    for a, b in zip(got, (kc, m[0], m[1], vc, m[2], m[3])):
        assert np.array_equal(a.view(np.uint8) if a.dtype == np.float16 else a,
                              b.view(np.uint8) if b.dtype == np.float16 else b)


def test_layout_hand_worked_positions():
    """tests/golden/layout_positions.json: bit positions derived by hand from the layout
    statement at the top of oracle/layout.py"""
    with open(os.path.join(GOLD, "layout_positions.json")) as f:
        gold = json.load(f)
    for g in gold["positions"]:
        fn = layout.k_code_bit if g["kind"] == "K" else layout.v_code_bit
        assert fn(g["slot"], g["channel"], g["bits"], g["D"]) == g["bit"], g


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_every_slot_owns_whole_bytes(bits, D):
    """a slot can be rewritten in place without touching its neighbours' bytes"""
    for fn in (layout.k_code_bit, layout.v_code_bit):
        owner = {}
        for t in range(16):
            for c in range(D):
                for bit in range(fn(t, c, bits, D), fn(t, c, bits, D) + bits):
                    assert owner.setdefault(bit // 8, t) == t
        assert len(owner) == 64 * layout.chunk_bytes(bits, D)
