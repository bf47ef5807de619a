"""Byte image of a KV page (test infrastructure; see oracle/__init__.py).

The oracle keeps codes unpacked; this module is the independent packer that turns one
(page, kv-head) worth of unpacked state into the exact bytes the device arena must hold,
so the two can be compared bit for bit.  The paper fixes no bit order (its only remark,
in "System Optimizations", is that two 2-bit tokens are padded into one 4-bit cell for
alignment, which thought-aware paging makes unnecessary: a block holds one thought type,
Sec. 5.2 "Block Table").  The layout below is this build's own, stated as formulas.

A page holds P = 16 slots; head_dim D in {64,128}; NG = D/32 groups; b in {2,4,8} bits.
Per (page, kv-head) there is one block of four regions, in this order:

    K codes : 64 chunks of CB = NG*b bytes          (chunk index L_K)
    K meta  : NG*4 units of eight binary16; unit group*4 + slot//4 holds the scales of its
              four slots (slot%4 = 0..3), then their four zero-points
    V codes : 64 chunks of CB bytes                  (chunk index L_V)
    V meta  : as K meta

Inside a chunk a code occupies b bits at bit offset  32*(f // FPH) + 16*h + b*(f % FPH),
FPH = 16/b, where (chunk, f, h) are

    K, slot t, channel c :  group = c//32, j = (c%32)//8, e = c%8
                            L_K = 16*j + t,  f = 4*group + e//2,  h = e%2
    V, slot t, channel c :  q = t//4, r = t%4, mb = c//16, m = c%16
                            L_V = 16*q + m,  f = (r//2)*(D/16) + mb,  h = r%2

(bit offsets count from the least significant bit of the chunk read as a little-endian
integer).  A page is n_kv_heads such blocks back to back; an arena is pages back to back.

The paper's own formats (formats.py) keep the code regions exactly as above (an E2M1 nibble, a
ternary code or an E4M3 byte is a 4-, 2- or 8-bit code like any other); only the meta regions
differ: one E4M3 scale byte per (slot, group of 16 channels), at byte  group16*16 + slot  of the
region (D/16 * 16 bytes), and no meta region at all for the 8-bit type, whose scale is per tensor.
"""
import numpy as np

PAGE = 16


def chunk_bytes(bits, D):
    return (D // 32) * bits


def block_bytes(bits, D):
    return 2 * (64 * chunk_bytes(bits, D) + PAGE * (D // 32) * 4)


def page_bytes(bits, D, n_kv_heads):
    return n_kv_heads * block_bytes(bits, D)


def region_offsets(bits, D):
    """byte offsets of (K codes, K meta, V codes, V meta) inside a block"""
    cb = 64 * chunk_bytes(bits, D)
    mb = PAGE * (D // 32) * 4
    return 0, cb, cb + mb, 2 * cb + mb


def k_code_bit(t, c, bits, D):
    fph = 16 // bits
    group, j, e = c // 32, (c % 32) // 8, c % 8
    lane = 16 * j + t
    f, h = 4 * group + e // 2, e % 2
    return 8 * chunk_bytes(bits, D) * lane + 32 * (f // fph) + 16 * h + bits * (f % fph)


def v_code_bit(t, c, bits, D):
    fph = 16 // bits
    q, r, mb, m = t // 4, t % 4, c // 16, c % 16
    lane = 16 * q + m
    f, h = (r // 2) * (D // 16) + mb, r % 2
    return 8 * chunk_bytes(bits, D) * lane + 32 * (f // fph) + 16 * h + bits * (f % fph)


def _pack_codes(codes, bits, D, bitfn):
    """codes: uint8 [..., 16, D] -> uint8 [..., 64*CB].  Every code lands on b bits of its
    own, so OR-ing the shifted codes of one dword equals summing them."""
    lead = codes.shape[:-2]
    t, c = np.meshgrid(np.arange(PAGE), np.arange(D), indexing="ij")
    pos = bitfn(t, c, bits, D).reshape(-1)
    order = np.argsort(pos, kind="stable")
    per_dword = 32 // bits
    spos = pos[order]
    assert np.array_equal(spos, np.arange(spos.size) * bits), "layout must tile the region exactly"
    flat = codes.reshape(lead + (PAGE * D,))[..., order].astype(np.uint32)
    shifted = flat << (spos % 32).astype(np.uint32)
    dwords = shifted.reshape(lead + (spos.size // per_dword, per_dword)).sum(axis=-1, dtype=np.uint32)
    return np.ascontiguousarray(dwords).view(np.uint8)          # host is little-endian


def _pack_meta(scale, zp):
    """scale, zp: float16 [..., 16, NG] -> uint8 [..., 16*NG*4]: for every group, for every
    quad of slots, the four scales then the four zero-points"""
    scale = np.asarray(scale, dtype=np.float16)
    zp = np.asarray(zp, dtype=np.float16)
    lead, ng = scale.shape[:-2], scale.shape[-1]
    units = np.empty(lead + (ng, 4, 2, 4), dtype=np.float16)
    for g in range(ng):
        for q in range(4):
            units[..., g, q, 0, :] = scale[..., 4 * q:4 * q + 4, g]
            units[..., g, q, 1, :] = zp[..., 4 * q:4 * q + 4, g]
    return np.ascontiguousarray(units).reshape(lead + (ng * 32,)).view(np.uint8)


def pack_page_head(k_codes, k_scale, k_zp, v_codes, v_scale, v_zp, bits):
    """k_codes, v_codes: uint8 [..., 16, D]; *_scale, *_zp: float16 [..., 16, D/32].
    Returns the uint8 [..., block_bytes] image of each (page, kv-head)."""
    D = k_codes.shape[-1]
    return np.concatenate([
        _pack_codes(k_codes, bits, D, k_code_bit), _pack_meta(k_scale, k_zp),
        _pack_codes(v_codes, bits, D, v_code_bit), _pack_meta(v_scale, v_zp)], axis=-1)


def block_bytes_fp(bits, D):
    return 2 * (64 * chunk_bytes(bits, D) + (0 if bits == 8 else PAGE * (D // 16)))


def _pack_meta_fp(scale_codes):
    """E4M3 scale codes uint8 [..., 16, D/16] -> uint8 [..., D/16 * 16]: byte group16*16 + slot"""
    sc = np.asarray(scale_codes, dtype=np.uint8)
    return np.ascontiguousarray(np.swapaxes(sc, -1, -2)).reshape(sc.shape[:-2] + (sc.shape[-1] * PAGE,))


def pack_page_head_fp(k_codes, k_scale_codes, v_codes, v_scale_codes, bits):
    """the paper's formats: k_codes, v_codes uint8 [..., 16, D]; *_scale_codes uint8 [..., 16, D/16] (ignored at 8 bits).
    Returns the uint8 [..., block_bytes_fp] image of each (page, kv-head)."""
    D = k_codes.shape[-1]
    parts = [_pack_codes(k_codes, bits, D, k_code_bit)]
    if bits != 8:
        parts.append(_pack_meta_fp(k_scale_codes))
    parts.append(_pack_codes(v_codes, bits, D, v_code_bit))
    if bits != 8:
        parts.append(_pack_meta_fp(v_scale_codes))
    return np.concatenate(parts, axis=-1)
