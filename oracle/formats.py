"""The paper's own number formats (test infrastructure; see oracle/__init__.py).

Sec. 4.2 ("Think Before You Quantize") and the appendix "Quantization Data Formats" give the
three precisions as floating-point formats: FP8 (E4M3: 1 sign, 4 exponent, 3 mantissa bits)
with one binary32 scale per tensor; NVFP4 (E2M1: 1 sign, 2 exponent, 1 mantissa bit) with one
E4M3 scale per group of 16; ternary (two bits for {-1, 0, +1}; the fourth code is a negative
zero and reads as 0) with one E4M3 scale per group of 16.

This module is the definition of those formats written out (decode tables from the bit
fields, encoders that round to the nearest representable value, ties to the even code, and
saturate), plus the group quantisers built on them.

Readings where the paper is silent:
  * E4M3 is the finite-only variant used for FP8 inference (bias 7, largest value 448, the
    code S.1111.111 is NaN, no infinities); E2M1 has bias 1 and no special codes
    (0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives);
  * ternary code = sign bit, magnitude bit: 0 -> 0, 1 -> +1, 2 -> -0 (reads 0), 3 -> -1;
  * a group's scale is amax / qmax (qmax = 6 for E2M1, 1 for ternary) rounded UP to the next
    E4M3 value (at least 2^-9, the smallest one, for any group that is not all zeros; 448 at
    most, beyond which elements saturate), so that the largest element never saturates by more
    than rounding; a group of zeros has scale 0 and decodes to zeros; no second, per-tensor
    scale sits under the E4M3 group scales (the paper names one only for FP8);
  * the per-tensor binary32 scale of FP8 comes from calibration and is an input here;
  * groups run along head_dim inside one token, for keys and values alike (16 consecutive
    channels).  The paper quantises keys per channel over groups of g tokens held back in a
    full-precision buffer; a slot that is refilled in place would then inherit a scale fitted
    to other tokens, and the paper does not say how slot reuse and per-channel groups go
    together.  Token-local groups keep every token self-contained, as the integer formats of
    this build already are.
"""
import numpy as np

GROUP16 = 16
E4M3_MAX = 448.0
E2M1_MAX = 6.0


def _decode_table(exp_bits, man_bits, bias, nan_code=None):
    """value of every code of a sign / exponent / mantissa format with gradual underflow"""
    n = 1 << (1 + exp_bits + man_bits)
    out = np.zeros(n, dtype=np.float64)
    for code in range(n):
        sign = -1.0 if code >> (exp_bits + man_bits) else 1.0
        e = (code >> man_bits) & ((1 << exp_bits) - 1)
        m = code & ((1 << man_bits) - 1)
        if e == 0:
            mag = m / (1 << man_bits) * 2.0 ** (1 - bias)
        else:
            mag = (1.0 + m / (1 << man_bits)) * 2.0 ** (e - bias)
        out[code] = sign * mag
    if nan_code is not None:
        out[nan_code] = np.nan
        out[nan_code | (n >> 1)] = np.nan
    return out


E4M3_VALUES = _decode_table(4, 3, 7, nan_code=0x7F)      # [256]
E2M1_VALUES = _decode_table(2, 1, 1)                     # [16]
TERNARY_VALUES = np.array([0.0, 1.0, 0.0, -1.0])         # code 2 is the negative zero


def _encode_nearest(x, magnitudes):
    """index of the magnitude nearest |x| (ties to the even index), saturating at the largest; magnitudes ascending from 0"""
    a = np.abs(np.asarray(x, dtype=np.float64))
    hi = np.searchsorted(magnitudes, a, side="left")          # first magnitude >= a
    hi = np.clip(hi, 0, len(magnitudes) - 1)
    lo = np.clip(hi - 1, 0, len(magnitudes) - 1)
    d_lo, d_hi = a - magnitudes[lo], magnitudes[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    idx = np.where(take_hi, hi, lo)
    idx = np.where(a >= magnitudes[-1], len(magnitudes) - 1, idx)
    return idx


_E4M3_MAG = E4M3_VALUES[:0x7F]          # codes 0 .. 0x7E: ascending magnitudes 0 .. 448
_E2M1_MAG = E2M1_VALUES[:8]


def e4m3_encode(x):
    """nearest E4M3 code (ties to even, |x| > 448 saturates to 448; NaN -> 0x7F)"""
    x = np.asarray(x, dtype=np.float64)
    code = _encode_nearest(np.nan_to_num(x, nan=0.0), _E4M3_MAG).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)


def e4m3_decode(code):
    return E4M3_VALUES[np.asarray(code, dtype=np.uint8)]


def e4m3_encode_up(x):
    """smallest E4M3 value >= x for x >= 0 (saturating at 448): a scale that never under-covers"""
    x = np.asarray(x, dtype=np.float64)
    idx = np.searchsorted(_E4M3_MAG, x, side="left")
    return np.clip(idx, 0, len(_E4M3_MAG) - 1).astype(np.uint8)


def e2m1_encode(x):
    """nearest E2M1 code (ties to even, saturating at +-6); four bits, sign in bit 3"""
    x = np.asarray(x, dtype=np.float64)
    code = _encode_nearest(x, _E2M1_MAG).astype(np.uint8)
    return np.where(np.signbit(x) & (code != 0), code | 8, code).astype(np.uint8)


def e2m1_decode(code):
    return E2M1_VALUES[np.asarray(code, dtype=np.uint8) & 15]


def ternary_encode(x):
    """-1, 0 or +1, whichever is nearest (|x| = 0.5 goes to 0, the even choice); two bits, sign in bit 1"""
    x = np.asarray(x, dtype=np.float64)
    mag = (np.abs(x) > 0.5).astype(np.uint8)
    return np.where((x < 0) & (mag == 1), np.uint8(3), mag).astype(np.uint8)


def ternary_decode(code):
    return TERNARY_VALUES[np.asarray(code, dtype=np.uint8) & 3]


# ----------------------------------------------------------------------- group quantisers
def _groups(x):
    x = np.asarray(x, dtype=np.float64)
    if x.shape[-1] % GROUP16:
        raise ValueError("last dimension must be a multiple of 16")
    return x.reshape(x.shape[:-1] + (x.shape[-1] // GROUP16, GROUP16))


def _group_scale(xg, qmax):
    amax = np.abs(xg).max(axis=-1)
    code = e4m3_encode_up(amax / qmax)
    return code, e4m3_decode(code)


def nvfp4_quantize(x):
    """x [..., D] -> (codes uint8 [..., D] in 0..15, scale codes uint8 [..., D/16] (E4M3))"""
    xg = _groups(x)
    scode, s = _group_scale(xg, E2M1_MAX)
    ratio = np.divide(xg, s[..., None], out=np.zeros_like(xg), where=s[..., None] > 0)
    return e2m1_encode(ratio).reshape(np.shape(x)), scode


def nvfp4_dequantize(codes, scale_codes):
    cg = _groups(e2m1_decode(codes))
    return (cg * e4m3_decode(scale_codes)[..., None]).reshape(np.shape(codes))


def ternary_quantize(x):
    """x [..., D] -> (codes uint8 [..., D] in {0, 1, 3}, scale codes uint8 [..., D/16] (E4M3))"""
    xg = _groups(x)
    scode, s = _group_scale(xg, 1.0)
    ratio = np.divide(xg, s[..., None], out=np.zeros_like(xg), where=s[..., None] > 0)
    return ternary_encode(ratio).reshape(np.shape(x)), scode


def ternary_dequantize(codes, scale_codes):
    cg = _groups(ternary_decode(codes))
    return (cg * e4m3_decode(scale_codes)[..., None]).reshape(np.shape(codes))


def fp8_quantize(x, tensor_scale):
    """E4M3 codes of x / tensor_scale (one binary32 scale for the whole tensor, from calibration)"""
    return e4m3_encode(np.asarray(x, dtype=np.float64) / float(np.float32(tensor_scale)))


def fp8_dequantize(codes, tensor_scale):
    return e4m3_decode(codes) * float(np.float32(tensor_scale))
