"""Numpy reading of the tile layout, written from its specification (not from the kernels).

``tiles_to_canonical`` turns the codes / radii tiles of one head plane into
canonical 62-byte records, so that what the encode kernel stores can be
compared byte for byte with the oracle's records without going through the
library's own export kernel.
"""
import numpy as np

OFF_L1A, OFF_L1B, OFF_G6, OFF_C4 = 0, 1024, 2048, 2816
CODE_BYTES, RADII = 2944, 512


def _bits(buf, bit, width):
    """buf: uint8 [..., nbytes]; little-endian bit string; returns the field as int."""
    byte, sh = bit // 8, bit % 8
    v = buf[..., byte].astype(np.uint32) | (buf[..., byte + 1].astype(np.uint32) << 8)
    return (v >> sh) & ((1 << width) - 1)


def block_fields(kind, codes, radii, tau, b):
    """codes: uint8 [T, 2944], radii: uint16 [T, 512] -> (l1 32-bit, g6[2], c4, radius) arrays over tiles."""
    i = tau >> 4
    if kind == 0:  # key tile: lane = 16*quarter + (tau mod 16), chunk i
        m, gk, beta = tau & 15, b >> 1, b & 1
        lam = 16 * gk + m
        l1_at = (OFF_L1A if i < 2 else OFF_L1B) + lam * 16 + (i & 1) * 8 + beta * 4
        l1 = codes[:, l1_at : l1_at + 4].copy().view(np.uint32)[:, 0]
        gbit = (OFF_G6 + lam * 12) * 8 + 24 * i + 12 * beta
        g6 = [_bits(codes, gbit, 6), _bits(codes, gbit + 6, 6)]
        c4 = _bits(codes, (OFF_C4 + lam * 2) * 8 + 4 * i + 2 * beta, 2)
        rad = radii[:, lam * 8 + 2 * i + beta]
    else:  # value tile: lane = 16*g + half-block, slot s
        g, e = (tau >> 2) & 3, tau & 3
        s = 4 * i + e
        halves, g6 = [], []
        for h in range(2):
            lam = 16 * g + 2 * b + h
            at = (OFF_L1A if s < 8 else OFF_L1B) + lam * 16 + (s & 7) * 2
            halves.append(codes[:, at].astype(np.uint32) | (codes[:, at + 1].astype(np.uint32) << 8))
            g6.append(_bits(codes, (OFF_G6 + lam * 12) * 8 + 6 * s, 6))
        l1 = halves[0] | (halves[1] << 16)
        c4 = _bits(codes, (OFF_C4 + (g * 8 + b) * 4) * 8 + 2 * s, 2)
        rad = radii[:, (g * 8 + b) * 16 + s]
    return l1, g6, c4, rad


def tiles_to_canonical(kind, codes, radii, n_tokens):
    """codes uint8 [T, 2944], radii uint16 [T, 512] of one head plane -> records uint8 [n_tokens, 62]."""
    codes = np.ascontiguousarray(codes)
    # one spare byte so that 2-byte windows at the very end stay in range
    codes = np.concatenate([codes, np.zeros((codes.shape[0], 2), np.uint8)], axis=1)
    radii = np.ascontiguousarray(radii).view(np.uint16)
    T = codes.shape[0]
    rec = np.zeros((T, 64, 62), dtype=np.uint8)
    for tau in range(64):
        for b in range(8):
            l1, g6, c4, rad = block_fields(kind, codes, radii, tau, b)
            for k in range(4):
                even = (l1 >> (8 * k)) & 15
                odd = (l1 >> (8 * k + 4)) & 15
                rec[:, tau, 4 * b + k] = (even << 4) | odd
            c2 = [g6[0] >> 4, g6[0] & 3, g6[1] >> 4, g6[1] & 3]
            rec[:, tau, 32 + b] = (c2[0] << 6) | (c2[1] << 4) | (c2[2] << 2) | c2[3]
            c3 = [(g6[0] >> 2) & 3, (g6[1] >> 2) & 3]
            for h in range(2):
                j = 2 * b + h
                rec[:, tau, 40 + j // 4] |= (c3[h] << (6 - 2 * (j & 3))).astype(np.uint8)
            rec[:, tau, 44 + b // 4] |= (c4 << (6 - 2 * (b & 3))).astype(np.uint8)
            rec[:, tau, 46 + 2 * b] = rad & 0xFF
            rec[:, tau, 47 + 2 * b] = rad >> 8
    return rec.reshape(T * 64, 62)[:n_tokens]


def tiles_to_canonical_deep(kind, codes, top, n_tokens):
    """Full-depth caches: codes uint8 [T, 2944] as above; the radius plane holds one 32-bit word per
    token (top: [T, 128] 16-bit halves = [T, 64] little-endian words, word tau = radius << 16 | upper
    codes) -> records uint8 [n_tokens, 50]: bytes 0..45 as in the 62-byte record, then the word."""
    T = np.ascontiguousarray(codes).shape[0]
    words = np.ascontiguousarray(top).view(np.uint16).reshape(T, 64, 2)   # [.., 0] low half: codes, [.., 1]: radius
    base = tiles_to_canonical(kind, codes, np.zeros((T, RADII), np.uint16), T * 64).reshape(T, 64, 62)
    rec = np.zeros((T, 64, 50), dtype=np.uint8)
    rec[:, :, :46] = base[:, :, :46]
    rec[:, :, 46] = words[:, :, 0] & 0xFF
    rec[:, :, 47] = words[:, :, 0] >> 8
    rec[:, :, 48] = words[:, :, 1] & 0xFF
    rec[:, :, 49] = words[:, :, 1] >> 8
    return rec.reshape(T * 64, 50)[:n_tokens]
