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
