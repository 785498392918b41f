"""Numpy reading and writing of the tile layout, written from its specification (the comment at
the top of paper_2502_02617_amd/csrc/pq_layout.h), not from the kernels.

``tiles_to_canonical`` turns the codes / radii tiles of one head plane into canonical 62-byte
records, so that what the encode kernel stores can be compared byte for byte with the oracle's
records without going through the library's own export kernel.  ``canonical_to_tiles`` is its
inverse: it lays canonical records (the oracle's) out as tiles, so that the attention kernels can
be run on a cache that no library kernel has written.

Specification, restated.  A block of 16 coordinates has four 10-bit quarter indices
Q_j = c1_{2j+1} << 6 | c2_j << 4 | c1_{2j}, one 6-bit block index B = c4 << 4 | c3_0 << 2 | c3_1 and a
binary16 radius.  Bit strings are little endian.
  key tile:   token tau owns a 368-bit string, block b at bit 46 b: Q_0 | Q_1 << 10 | Q_2 << 20 | Q_3 << 30 |
              B << 40; string bytes 0..15 at tile byte 16 tau, 16..31 at 1024 + 16 tau, 32..43 at
              2048 + 12 tau, 44..45 at 2816 + 2 tau; radius of block b at half 8 tau + b.
  value tile: token tau = 16 i + 4 g + e is slot s = 4 i + e of the lanes 16 g + 2 b + h (h = 0, 1: the halves
              of block b); lane lam owns a 320-bit string, slot s at bit 20 s: Q_{2h} | Q_{2h+1} << 10; string
              bytes 0..15 at tile byte 16 lam, 16..31 at 1024 + 16 lam, 32..39 at 2048 + 8 lam; the block
              indices of (g, b) are a 96-bit string at tile byte 2560 + 12 (8 g + b), slot s at bit 6 s; radius
              of slot s of (g, b) at half 16 (8 g + b) + s.
"""
import numpy as np

CODE_BYTES, RADII = 2944, 512
KEY, VALUE_Q, VALUE_B = 0, 1, 2


def string_byte(stype, owner, k):
    """tile byte holding byte k of a string"""
    if stype == VALUE_B:
        return 2560 + 12 * owner + k
    if k < 16:
        return 16 * owner + k
    if k < 32:
        return 1024 + 16 * owner + (k - 16)
    if stype == KEY:
        return 2048 + 12 * owner + (k - 32) if k < 44 else 2816 + 2 * owner + (k - 44)
    return 2048 + 8 * owner + (k - 32)


def get_bits(codes, stype, owner, bit, width):
    """codes uint8 [T, 2944] -> the field (width <= 16) as uint32 [T]; the bytes of a string are looked up one by one"""
    first, sh = divmod(bit, 8)
    v = np.zeros(codes.shape[0], dtype=np.uint32)
    for n in range((sh + width + 7) // 8):
        v |= codes[:, string_byte(stype, owner, first + n)].astype(np.uint32) << np.uint32(8 * n)
    return (v >> np.uint32(sh)) & np.uint32((1 << width) - 1)


def put_bits(codes, stype, owner, bit, width, value):
    """writes value (uint32 [T], width <= 16) into codes uint8 [T, 2944], byte piece by byte piece"""
    first, sh = divmod(bit, 8)
    v = (value.astype(np.uint32) & np.uint32((1 << width) - 1)) << np.uint32(sh)
    m = ((1 << width) - 1) << sh
    for n in range((sh + width + 7) // 8):
        at = string_byte(stype, owner, first + n)
        keep = 0xFF ^ ((m >> (8 * n)) & 0xFF)
        codes[:, at] = (codes[:, at] & np.uint8(keep)) | ((v >> np.uint32(8 * n)) & np.uint32(0xFF)).astype(np.uint8)


def block_places(kind, tau, b):
    """-> ([(stype, owner, bit) of Q_0..Q_3], (stype, owner, bit) of B, radius half)"""
    if kind == 0:
        return [(KEY, tau, 46 * b + 10 * j) for j in range(4)], (KEY, tau, 46 * b + 40), 8 * tau + b
    i, g, e = tau >> 4, (tau >> 2) & 3, tau & 3
    s = 4 * i + e
    q = [(VALUE_Q, 16 * g + 2 * b + (j >> 1), 20 * s + 10 * (j & 1)) for j in range(4)]
    return q, (VALUE_B, 8 * g + b, 6 * s), 16 * (8 * g + b) + s


def _codes_of_tile_fields(Q, B):
    """Q [T, 4], B [T] -> (c1 [T, 8], c2 [T, 4], c3 [T, 2], c4 [T])"""
    c1 = np.stack([(Q[:, p >> 1] >> (6 * (p & 1))) & 15 for p in range(8)], axis=1)
    c2 = (Q >> 4) & 3
    c3 = np.stack([(B >> 2) & 3, B & 3], axis=1)
    return c1, c2, c3, B >> 4


def tiles_to_canonical(kind, codes, radii, n_tokens):
    """codes uint8 [T, 2944], radii uint16 [T, 512] of one head plane -> records uint8 [n_tokens, 62]."""
    codes = np.ascontiguousarray(codes)
    radii = np.ascontiguousarray(radii).view(np.uint16)
    T = codes.shape[0]
    rec = np.zeros((T, 64, 62), dtype=np.uint8)
    for tau in range(64):
        for b in range(8):
            qp, bp, rh = block_places(kind, tau, b)
            Q = np.stack([get_bits(codes, *p, 10) for p in qp], axis=1)
            B = get_bits(codes, *bp, 6)
            c1, c2, c3, c4 = _codes_of_tile_fields(Q, B)
            for k in range(4):
                rec[:, tau, 4 * b + k] = (c1[:, 2 * k] << 4) | c1[:, 2 * k + 1]
            rec[:, tau, 32 + b] = (c2[:, 0] << 6) | (c2[:, 1] << 4) | (c2[:, 2] << 2) | c2[:, 3]
            for h in range(2):
                j = 2 * b + h
                rec[:, tau, 40 + j // 4] |= (c3[:, h] << (6 - 2 * (j & 3))).astype(np.uint8)
            rec[:, tau, 44 + b // 4] |= (c4 << (6 - 2 * (b & 3))).astype(np.uint8)
            rad = radii[:, rh]
            rec[:, tau, 46 + 2 * b] = rad & 0xFF
            rec[:, tau, 47 + 2 * b] = rad >> 8
    return rec.reshape(T * 64, 62)[:n_tokens]


def _record_codes(rec):
    """rec uint8 [n, >=46] -> (c1 [n, 64], c2 [n, 32], c3 [n, 16], c4 [n, 8]) in coordinate order"""
    r = rec.astype(np.uint32)
    c1 = np.stack([r[:, :32] >> 4, r[:, :32] & 15], axis=2).reshape(-1, 64)
    four = lambda x: np.stack([(x >> 6) & 3, (x >> 4) & 3, (x >> 2) & 3, x & 3], axis=2).reshape(x.shape[0], -1)
    return c1, four(r[:, 32:40]), four(r[:, 40:44]), four(r[:, 44:46])


def canonical_to_tiles(kind, rec, n_tiles=None, fill=0):
    """rec uint8 [n, 62] (slots 0..n-1 of one head plane) -> (codes uint8 [T, 2944], radii uint16 [T, 512]).
    Slots beyond n keep `fill` in every code byte and radius."""
    codes, radii = canonical_to_tiles_planes(kind, rec[None], n_tiles, fill)
    return codes[0], radii[0]


def canonical_to_tiles_planes(kind, rec, n_tiles=None, fill=0):
    """The same for several head planes at once: rec uint8 [G, n, 62] -> (codes uint8 [G, T, 2944], radii uint16
    [G, T, 512]); one pass over the 64 slots of a tile serves the tiles of all planes."""
    G, n = rec.shape[0], rec.shape[1]
    Tp = (n + 63) // 64 if n_tiles is None else n_tiles      # tiles per plane
    assert Tp * 64 >= n
    T = G * Tp
    full = np.zeros((G, Tp * 64, 62), dtype=np.uint8)
    full[:, :n] = rec
    full = full.reshape(T * 64, 62)
    c1, c2, c3, c4 = _record_codes(full)
    rad = full[:, 46:62].astype(np.uint16)
    rad = (rad[:, 0::2] | (rad[:, 1::2] << 8)).reshape(T, 64, 8)
    c1, c2, c3, c4 = c1.reshape(T, 64, 64), c2.reshape(T, 64, 32), c3.reshape(T, 64, 16), c4.reshape(T, 64, 8)
    codes = np.full((T, CODE_BYTES), fill & 0xFF, dtype=np.uint8)
    radii = np.full((T, RADII), (fill & 0xFF) * 0x0101, dtype=np.uint16)
    for tau in range(64):
        # which tiles actually hold slot tau
        live = ((np.arange(T) % Tp) * 64 + tau) < n
        if not live.any():
            continue
        sub = codes[live]
        for b in range(8):
            qp, bp, rh = block_places(kind, tau, b)
            for j in range(4):
                Q = (c1[live, tau, 8 * b + 2 * j + 1] << 6) | (c2[live, tau, 4 * b + j] << 4) | c1[live, tau, 8 * b + 2 * j]
                put_bits(sub, *qp[j], 10, Q)
            B = (c4[live, tau, b] << 4) | (c3[live, tau, 2 * b] << 2) | c3[live, tau, 2 * b + 1]
            put_bits(sub, *bp, 6, B)
            radii[live, rh] = rad[live, tau, b]
        codes[live] = sub
    return codes.reshape(G, Tp, CODE_BYTES), radii.reshape(G, Tp, RADII)


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


def canonical_to_tiles_deep(kind, rec, n_tiles=None, fill=0):
    """rec uint8 [n, 50] -> (codes uint8 [T, 2944], top uint16 [T, 128]): the inverse of tiles_to_canonical_deep."""
    n = rec.shape[0]
    T = (n + 63) // 64 if n_tiles is None else n_tiles
    wide = np.zeros((n, 62), dtype=np.uint8)
    wide[:, :46] = rec[:, :46]
    codes, _ = canonical_to_tiles(kind, wide, T, fill)
    top = np.full((T * 64, 2), (fill & 0xFF) * 0x0101, dtype=np.uint16)
    r = rec.astype(np.uint16)
    top[:n, 0] = r[:, 46] | (r[:, 47] << 8)
    top[:n, 1] = r[:, 48] | (r[:, 49] << 8)
    return codes, top.reshape(T, 128)


def unpack_canonical(rec):
    """Canonical 62-byte records -> (codes int32 [n, 120]: the 64 level-1, 32 level-2, 16 level-3 and 8 level-4
    codes in coordinate order; radii uint16 [n, 8]).  Written from the record specification (bytes 0..31 level 1,
    two codes per byte, earlier code in the high nibble; 32..39 / 40..43 / 44..45 levels 2 / 3 / 4, four per byte,
    earlier code in the higher bits; 46..61 the radii, little endian)."""
    rec = np.ascontiguousarray(rec).reshape(-1, 62)
    c1, c2, c3, c4 = _record_codes(rec)
    r = rec[:, 46:62].astype(np.uint16)
    return np.concatenate([c1, c2, c3, c4], axis=1).astype(np.int32), (r[:, 0::2] | (r[:, 1::2] << 8)).astype(np.uint16)


def unpack_canonical_deep(rec, bits):
    """Full-depth 50-byte records -> (codes int32 [n, 127]: as above, then the 4 + 2 + 1 codes of levels 5, 6, 7 from
    the 16-bit word at bytes 46..47 (level-5 codes lowest, bits[l-5] bits each); radius uint16 [n] from bytes 48..49)."""
    rec = np.ascontiguousarray(rec).reshape(-1, 50)
    c1, c2, c3, c4 = _record_codes(rec)
    r = rec.astype(np.uint32)
    word = r[:, 46] | (r[:, 47] << 8)
    up, at = [], 0
    for count, b in ((4, bits[0]), (2, bits[1]), (1, bits[2])):
        for _ in range(count):
            up.append((word >> at) & ((1 << b) - 1))
            at += b
    radius = (r[:, 48] | (r[:, 49] << 8)).astype(np.uint16)
    return np.concatenate([c1, c2, c3, c4, np.stack(up, axis=1)], axis=1).astype(np.int32), radius
