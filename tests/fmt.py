"""Test-side readers of the partition record format (see include/bpc.h).

Written against the format description only; used to look inside payloads
produced by the oracle and by the GPU library.
"""
import numpy as np


def ru4(x):
    return (x + 3) // 4 * 4


def k_of(k_ratio, d):
    return min(d, max(1, int(np.floor(k_ratio * d))))


def dither_planes(levels):
    """Bit planes after the nibbles of a linear-dithering record: level bits 3, 4, 5."""
    planes = 0
    while (levels >> (3 + planes)) != 0:
        planes += 1
    return planes


def stride(kind, part_elems, k_ratio=0.0, levels=4):
    if kind == "identity":
        words = ru4(part_elems)
    elif kind == "sign":
        words = ru4((part_elems + 31) // 32)
    elif kind == "dither":
        words = ru4((part_elems + 7) // 8) + dither_planes(levels) * ru4((part_elems + 31) // 32)
    elif kind == "natdither":
        words = ru4((part_elems + 7) // 8)
    elif kind == "fp16":
        words = ru4((part_elems + 1) // 2)
    elif kind == "topk":
        words = 2 * ru4(k_of(k_ratio, part_elems))
    elif kind == "topk16":
        words = ru4(k_of(k_ratio, part_elems)) + ru4((k_of(k_ratio, part_elems) + 1) // 2)
    elif kind == "randk":
        words = ru4(k_of(k_ratio, part_elems))
    else:
        raise ValueError(kind)
    return 16 + 4 * words


def part_sizes(D, part_elems):
    return [min(part_elems, D - lo) for lo in range(0, D, part_elems)]


def record(payload, p, strd):
    return payload[p * strd:(p + 1) * strd]


def header_f32(rec):
    return rec[:4].view(np.float32)[0]


def header_u32(rec):
    return int(rec[:4].view(np.uint32)[0])


def sign_bits(rec, d):
    """-> (sigma, bool array of d sign bits, padding words as uint32)."""
    nw = (d + 31) // 32
    words = rec[16:16 + 4 * ru4(nw)].view(np.uint32)
    bits = np.unpackbits(words[:nw].view(np.uint8), bitorder="little")[:d].astype(bool)
    return header_f32(rec), bits, words


def dither_nibbles(rec, d):
    """-> (nu, sign bool[d], level uint8[d], words)."""
    nw = (d + 7) // 8
    words = rec[16:16 + 4 * ru4(nw)].view(np.uint32)
    by = words[:nw].view(np.uint8)
    nib = np.empty(2 * by.size, dtype=np.uint8)
    nib[0::2] = by & 0xF
    nib[1::2] = by >> 4
    nib = nib[:d]
    return header_f32(rec), (nib & 8) != 0, nib & 7, words


def dither_levels(rec, d, part_elems, levels):
    """-> (nu, sign bool[d], level uint8[d]) of a linear-dithering record with its bit planes."""
    nu, sgn, lvl, _ = dither_nibbles(rec, d)
    lvl = lvl.astype(np.uint8)
    off0 = 16 + 4 * ru4((part_elems + 7) // 8)
    pw = 4 * ru4((part_elems + 31) // 32)
    for t in range(dither_planes(levels)):
        words = rec[off0 + t * pw:off0 + t * pw + 4 * ((d + 31) // 32)].view(np.uint32)
        bits = np.unpackbits(words.view(np.uint8), bitorder="little")[:d]
        lvl |= (bits << (3 + t)).astype(np.uint8)
    return nu, sgn, lvl


def fp16_values(rec, d):
    """-> float16[d] of an FP16 record."""
    return rec[16:16 + 2 * d].view(np.float16)


def topk_entries(rec, k_cap):
    k = header_u32(rec)
    idx = rec[16:16 + 4 * k].view(np.int32)
    off = 16 + 4 * ru4(k_cap)
    val = rec[off:off + 4 * k].view(np.float32)
    return k, idx, val


def topk16_entries(rec, k_cap):
    k = header_u32(rec)
    idx = rec[16:16 + 4 * k].view(np.int32)
    off = 16 + 4 * ru4(k_cap)
    val = rec[off:off + 2 * k].view(np.float16)
    return k, idx, val


def randk_values(rec):
    k = header_u32(rec)
    return k, rec[16:16 + 4 * k].view(np.float32)


def defined_bytes(kind, d, k=0, k_cap=0, part_elems=0, levels=4):
    """Byte ranges of a record that the format defines for a partition of d elements."""
    if kind == "dither" and dither_planes(levels) > 0:
        off0 = 16 + 4 * ru4((part_elems + 7) // 8)
        pw = 4 * ru4((part_elems + 31) // 32)
        return [(0, 16 + 4 * ru4((d + 7) // 8))] + [(off0 + t * pw, off0 + t * pw + 4 * ru4((d + 31) // 32))
                                                    for t in range(dither_planes(levels))]
    if kind == "identity":
        return [(0, 16 + 4 * d)]
    if kind == "sign":
        return [(0, 16 + 4 * ru4((d + 31) // 32))]
    if kind == "fp16":
        return [(0, 16 + 4 * ru4((d + 1) // 2))]
    if kind in ("dither", "natdither"):
        return [(0, 16 + 4 * ru4((d + 7) // 8))]
    if kind == "topk":
        off = 16 + 4 * ru4(k_cap)
        return [(0, 16 + 4 * k), (off, off + 4 * k)]
    if kind == "topk16":
        off = 16 + 4 * ru4(k_cap)
        return [(0, 16 + 4 * k), (off, off + 4 * ru4((k + 1) // 2))]
    if kind == "randk":
        return [(0, 16 + 4 * k)]
    raise ValueError(kind)
