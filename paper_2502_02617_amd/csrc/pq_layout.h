/*
 * pq_layout.h -- in-tile bit layout of the packed PolarQuant cache.
 *
 * The paper fixes the bit budget (Section 4.1: per block of 16 coordinates
 * 8x4 + 4x2 + 2x2 + 1x2 = 46 code bits and one 16-bit radius) and that the
 * indices are packed into 8-bit units; the order inside the cache is this
 * library's choice, made so that a 64-lane wavefront loads a 64-token tile
 * with a handful of full-width coalesced loads and every lane finds exactly
 * the fields it consumes in its own registers.
 *
 * Per vector (d = 128): 8 blocks b = 0..7 of 16 rotated coordinates.
 * Per block, four fields:
 *   L1   32 bits: 8 level-1 codes; code of pair p (coordinates 2p, 2p+1 of
 *        the block) in bits [4p, 4p+4).  The low 16 bits belong to half-block
 *        0 (coordinates 0..7), the high 16 bits to half-block 1.
 *   G6   2 x 6 bits, one group per half-block h:
 *          bits [4,6) level-2 code of node 2h   (coordinates 8h+0..3)
 *          bits [2,4) level-3 code of node h    (coordinates 8h+0..7)
 *          bits [0,2) level-2 code of node 2h+1 (coordinates 8h+4..7)
 *   C4   2 bits: the level-4 code of the block
 *   R    16 bits: binary16 radius of the block
 *
 * A tile is 64 consecutive token slots tau = 0..63 of one head plane:
 * 2944 code bytes (planes L1a, L1b, G6, C4) + 512 radii.
 *
 * Key tiles (PQ_KEY).  Lane lam = 16*gk + m (gk = 0..3 the quarter of the
 * vector = blocks 2gk and 2gk+1, m = 0..15) owns the four chunks
 * i = 0..3, chunk i = quarter gk of token tau = 16*i + m:
 *   L1a  [64 lanes][16 B] at byte    0: chunk 0 then chunk 1, each
 *                                       {L1 of block 2gk, L1 of block 2gk+1}
 *   L1b  [64 lanes][16 B] at byte 1024: chunks 2 and 3
 *   G6   [64 lanes][12 B] at byte 2048: 96-bit little-endian string, chunk i at
 *                                       bits [24i, 24i+24): groups (block 2gk,
 *                                       h=0), (2gk, h=1), (2gk+1, 0), (2gk+1, 1)
 *                                       at bit 6*(2*beta + h)
 *   C4   [64 lanes][ 2 B] at byte 2816: chunk i at bits [4i, 4i+4): block 2gk in
 *                                       the low pair of bits, block 2gk+1 above
 *   radii[64 lanes][ 8 halves]        : chunk i at halves 2i (block 2gk), 2i+1
 *
 * Value tiles (PQ_VALUE).  Lane lam = 16*g + n (n = 2*b + h the half-block,
 * g = 0..3) owns half-block n of the 16 tokens tau = 16*i + 4*g + e, stored
 * in slot s = 4*i + e (i, e = 0..3):
 *   L1a  [64 lanes][16 B] at byte    0: slots 0..7, 16 bits each: the L1 half
 *                                       of half-block n
 *   L1b  [64 lanes][16 B] at byte 1024: slots 8..15
 *   G6   [64 lanes][12 B] at byte 2048: 96-bit string, slot s at bits [6s, 6s+6)
 *   C4   [4 g][8 blocks][4 B] at byte 2816: slot s at bits [2s, 2s+2)
 *   radii[4 g][8 blocks][16 halves]   : slot s at half s
 */
#ifndef PQ_LAYOUT_H
#define PQ_LAYOUT_H

#include <stdint.h>

#define PQL_TILE_TOKENS 64
#define PQL_CODE_BYTES 2944
#define PQL_RADII 512
#define PQL_OFF_L1A 0
#define PQL_OFF_L1B 1024
#define PQL_OFF_G6 2048
#define PQL_OFF_C4 2816

#if defined(__HIPCC__)
#define PQL_HD __host__ __device__ __forceinline__
#else
#define PQL_HD inline
#endif

/* Position of one block's fields inside a tile: byte offsets are relative to
 * the tile's code bytes, bit offsets relative to the start of the named plane
 * region. */
struct PqBlockPos {
    uint32_t l1_byte[2];   /* byte offset of the 16-bit L1 half of half-block 0 / 1 */
    uint32_t g6_bit[2];    /* absolute bit offset (from the tile's first code byte) of G6 of half-block 0 / 1 */
    uint32_t c4_bit;       /* absolute bit offset of C4 */
    uint32_t radius_half;  /* index of the radius inside the tile's 512 halves */
};

PQL_HD PqBlockPos pql_key_pos(int tau, int b)
{
    int i = tau >> 4, m = tau & 15, gk = b >> 1, beta = b & 1;
    int lam = 16 * gk + m;
    PqBlockPos p;
    uint32_t l1 = (uint32_t)((i < 2 ? PQL_OFF_L1A : PQL_OFF_L1B) + lam * 16 + (i & 1) * 8 + beta * 4);
    p.l1_byte[0] = l1;
    p.l1_byte[1] = l1 + 2;
    uint32_t g = (uint32_t)((PQL_OFF_G6 + lam * 12) * 8 + 24 * i + 12 * beta);
    p.g6_bit[0] = g;
    p.g6_bit[1] = g + 6;
    p.c4_bit = (uint32_t)((PQL_OFF_C4 + lam * 2) * 8 + 4 * i + 2 * beta);
    p.radius_half = (uint32_t)(lam * 8 + 2 * i + beta);
    return p;
}

PQL_HD PqBlockPos pql_value_pos(int tau, int b)
{
    int i = tau >> 4, g = (tau >> 2) & 3, e = tau & 3, s = 4 * i + e;
    PqBlockPos p;
    for (int h = 0; h < 2; ++h) {
        int lam = 16 * g + 2 * b + h;
        p.l1_byte[h] = (uint32_t)((s < 8 ? PQL_OFF_L1A : PQL_OFF_L1B) + lam * 16 + (s & 7) * 2);
        p.g6_bit[h] = (uint32_t)((PQL_OFF_G6 + lam * 12) * 8 + 6 * s);
    }
    p.c4_bit = (uint32_t)((PQL_OFF_C4 + (g * 8 + b) * 4) * 8 + 2 * s);
    p.radius_half = (uint32_t)((g * 8 + b) * 16 + s);
    return p;
}

PQL_HD PqBlockPos pql_pos(int kind, int tau, int b)
{
    return kind == 0 ? pql_key_pos(tau, b) : pql_value_pos(tau, b);
}

/* Fields of one block, unpacked. */
struct PqBlockFields {
    uint32_t l1;      /* 8 level-1 codes, pair p in bits [4p,4p+4) */
    uint32_t g6[2];   /* per half-block: [c2(2h) | c3(h) | c2(2h+1)] */
    uint32_t c4;
    uint16_t radius;  /* binary16 bits */
};

/* Read `width` (<= 9) bits at absolute bit offset `bit` of a byte buffer;
 * touches the byte holding the first bit and the one after it. */
PQL_HD uint32_t pql_get_bits(const uint8_t *base, uint32_t bit, int width)
{
    uint32_t byte = bit >> 3, sh = bit & 7;
    uint32_t v = (uint32_t)base[byte] | ((uint32_t)base[byte + 1] << 8);
    return (v >> sh) & ((1u << width) - 1u);
}

/* Generic (slow) reader used by DeQuant and the canonical export.  radii == NULL: the
 * radius field is left zero (caches whose radius plane is not made of block radii). */
PQL_HD PqBlockFields pql_read_block(int kind, const uint8_t *codes, const uint16_t *radii, int tau, int b)
{
    PqBlockPos p = pql_pos(kind, tau, b);
    PqBlockFields f;
    uint32_t lo = (uint32_t)codes[p.l1_byte[0]] | ((uint32_t)codes[p.l1_byte[0] + 1] << 8);
    uint32_t hi = (uint32_t)codes[p.l1_byte[1]] | ((uint32_t)codes[p.l1_byte[1] + 1] << 8);
    f.l1 = lo | (hi << 16);
    /* a G6 read touches one byte past its first byte; the G6 plane ends at
       byte 2816 < 2944, so the window stays inside the tile.  C4 fields sit
       at even bit offsets and never straddle a byte. */
    f.g6[0] = pql_get_bits(codes, p.g6_bit[0], 6);
    f.g6[1] = pql_get_bits(codes, p.g6_bit[1], 6);
    {
        uint32_t byte = p.c4_bit >> 3, sh = p.c4_bit & 7;
        f.c4 = ((uint32_t)codes[byte] >> sh) & 3u;
    }
    f.radius = radii ? radii[p.radius_half] : (uint16_t)0;
    return f;
}

#endif /* PQ_LAYOUT_H */
