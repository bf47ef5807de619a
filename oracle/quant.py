"""Reference group quantizer (test infrastructure; see oracle/__init__.py).

Follows the paper's appendix section "Group Quantization": a tensor is cut into groups of
g consecutive entries that share one scale "and optionally zero-point"; codes are the
rounded ratio of the entry to the group scale, the scale being the group's range divided
by 2^b - 1.  The printed formula carries no minimum / zero-point; the reading used here is
the asymmetric round-to-nearest form (KIVI style, which the paper follows for its fused
dequantisation): zero-point = group minimum, scale = (max - min) / (2^b - 1), both stored
as IEEE binary16, groups of 32 along head_dim, so every token quantises on its own.
The bit width b comes from the thought class of the token (Problem "Thought-Adaptive
Quantization", Sec. 4.2: psi maps a thought type to a precision in {2,4,8}).

Arithmetic is specified to the operation so that an independent implementation can match
it bit for bit (inputs are binary16 / bfloat16 / binary32 values widened exactly to
binary32; every operation below is one IEEE binary32 operation, round-to-nearest-even):

    mn  = min(x), mx = max(x)                      over the 32 entries of the group
    zp  = f16(mn + 0.0)                            (+0.0 turns a -0.0 minimum into +0.0)
    s32 = (mx - mn) / (2^b - 1)
    s   = f16(s32); if f32(s) < s32: s = next binary16 above s      (so (2^b-1)*s >= range)
    c_i = clamp(rint((x_i - f32(zp)) / f32(s)), 0, 2^b - 1)          (s == 0: c_i = 0)

rint is round-half-to-even.  NaN / Inf inputs and ranges that overflow binary16 are
outside the supported domain.  Dequantisation is  x^_i = f32(zp) + c_i * f32(s).
"""
import numpy as np

GROUP = 32


def quantize_groups(x, bits):
    """x: float array [..., D] with D % 32 == 0 (values already exactly representable in
    binary32).  Returns (codes uint8 [..., D], scale float16 [..., D/32], zp float16 [..., D/32])."""
    if bits not in (2, 4, 8):
        raise ValueError("bits must be 2, 4 or 8")
    x = np.asarray(x, dtype=np.float32)
    if x.shape[-1] % GROUP:
        raise ValueError("last dimension must be a multiple of 32")
    xg = x.reshape(x.shape[:-1] + (x.shape[-1] // GROUP, GROUP))
    qmax = np.float32((1 << bits) - 1)
    mn = xg.min(axis=-1)
    mx = xg.max(axis=-1)
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        zp = (mn + np.float32(0.0)).astype(np.float16)
        s32 = ((mx - mn) / qmax).astype(np.float32)
        s = s32.astype(np.float16)
        low = s.astype(np.float32) < s32
        sb = s.view(np.uint16).copy()
        sb[low] += 1                      # positive binary16: next value up is bits + 1
        s = sb.view(np.float16)
        zf = zp.astype(np.float32)[..., None]
        sf = s.astype(np.float32)[..., None]
        diff = (xg - zf).astype(np.float32)
        ratio = np.where(sf > 0, diff / np.where(sf > 0, sf, np.float32(1.0)), np.float32(0.0)).astype(np.float32)
        c = np.rint(ratio)
        c = np.clip(c, np.float32(0.0), qmax)
    codes = c.astype(np.uint8).reshape(x.shape)
    return codes, s, zp


def dequantize(codes, scale, zp, dtype=np.float64):
    """x^ = zp + code * scale, evaluated in `dtype` from the stored binary16 scale / zero-point."""
    codes = np.asarray(codes)
    D = codes.shape[-1]
    cg = codes.reshape(codes.shape[:-1] + (D // GROUP, GROUP)).astype(dtype)
    out = np.asarray(zp).astype(dtype)[..., None] + cg * np.asarray(scale).astype(dtype)[..., None]
    return out.reshape(codes.shape)
