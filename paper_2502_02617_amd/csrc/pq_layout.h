/*
 * pq_layout.h -- in-tile bit layout of the packed PolarQuant cache.
 *
 * The paper fixes the bit budget (Section 4.1: per block of 16 coordinates
 * 8x4 + 4x2 + 2x2 + 1x2 = 46 code bits and one 16-bit radius) and that the
 * indices are packed into 8-bit units; the order inside the cache is this
 * library's choice.  It is made for the attention kernel, which rebuilds keys
 * and values from lookup tables: the codes of a block are stored as the table
 * indices the kernel uses, so that an index costs it one shift and one mask.
 *
 * Per vector (d = 128): 8 blocks b = 0..7 of 16 rotated coordinates.  With
 * c1_p the level-1 code of pair p = 0..7 (coordinates 2p, 2p+1 of the block),
 * c2_j the level-2 code of node j = 0..3 (coordinates 4j..4j+3), c3_h the
 * level-3 code of node h = 0, 1 (coordinates 8h..8h+7) and c4 the level-4
 * code, a block has six fields:
 *   Q_j  10 bits, j = 0..3 ("quarter index"): c1_{2j+1} << 6 | c2_j << 4 | c1_{2j}
 *        -- everything below level 3 of the four coordinates 4j..4j+3; its low six bits
 *        (c2_j, c1_{2j}) select the first pair of the quarter, its high six bits
 *        (c1_{2j+1}, c2_j) the second
 *   B     6 bits ("block index"): c4 << 4 | c3_0 << 2 | c3_1
 *   R    16 bits: binary16 radius of the block
 *
 * A tile is 64 consecutive token slots tau = 0..63 of one head plane:
 * 2944 code bytes + 512 radii (exactly 62 bytes per token).  All bit strings
 * below are little endian: bit p of a string is bit p & 7 of its byte p >> 3.
 *
 * Key tiles (PQ_KEY): one lane per token.  Token tau has a 368-bit code string,
 *   block b at bits [46 b, 46 b + 46): Q_0 | Q_1 << 10 | Q_2 << 20 | Q_3 << 30 | B << 40.
 *   Its 46 bytes are spread over four planes so that a wavefront loads them
 *   with full-width coalesced requests:
 *     bytes  0..15 at tile byte    0 + 16 tau   (plane KP0 [64][16])
 *     bytes 16..31 at tile byte 1024 + 16 tau   (plane KP1 [64][16])
 *     bytes 32..43 at tile byte 2048 + 12 tau   (plane KP2 [64][12])
 *     bytes 44..45 at tile byte 2816 +  2 tau   (plane KP3 [64][ 2])
 *   radii [64 tau][8 b]: the radius of block b of token tau at half 8 tau + b.
 *
 * Value tiles (PQ_VALUE): lane lam = 16 g + n (g = 0..3, n = 2 b + h the
 *   half-block) owns half-block n of the 16 tokens tau = 16 i + 4 g + e, kept in
 *   slot s = 4 i + e (i, e = 0..3).
 *   Lane lam has a 320-bit string, slot s at bits [20 s, 20 s + 20):
 *   Q_{2h} | Q_{2h+1} << 10.  Its 40 bytes:
 *     bytes  0..15 at tile byte    0 + 16 lam   (plane VP0 [64][16])
 *     bytes 16..31 at tile byte 1024 + 16 lam   (plane VP1 [64][16])
 *     bytes 32..39 at tile byte 2048 +  8 lam   (plane VP2 [64][ 8])
 *   The block indices of the 16 slots of (g, b) form a 96-bit string at tile byte
 *   2560 + 12 (8 g + b) (plane VB [4 g][8 b][12]), slot s at bits [6 s, 6 s + 6);
 *   both lanes of the block read it.
 *   radii [4 g][8 b][16 s]: slot s of (g, b) at half 16 (8 g + b) + s.
 */
#ifndef PQ_LAYOUT_H
#define PQ_LAYOUT_H

#include <stdint.h>

#define PQL_TILE_TOKENS 64
#define PQL_CODE_BYTES 2944
#define PQL_RADII 512
/* planes of 16, 16, 12 (keys) or 8 (values) bytes per lane, then the keys' 2-byte plane / the values' block-index plane */
#define PQL_OFF_P0 0
#define PQL_OFF_P1 1024
#define PQL_OFF_P2 2048
#define PQL_OFF_KP3 2816
#define PQL_OFF_VB 2560
#define PQL_BLOCK_BITS 46 /* bits of a block in a key token's string */
#define PQL_SLOT_BITS 20  /* bits of a slot in a value lane's string */

#if defined(__HIPCC__)
#define PQL_HD __host__ __device__ __forceinline__
#else
#define PQL_HD inline
#endif

/* A bit string of the layout: which one, and whose. */
enum { PQL_STR_KEY = 0, PQL_STR_VALUE_Q = 1, PQL_STR_VALUE_B = 2 };
struct PqString {
    int type;
    int owner; /* key: token tau; value Q: lane lam; value B: 8 g + b */
};

/* tile byte that holds byte k of the string */
PQL_HD uint32_t pql_string_byte(PqString s, int k)
{
    if (s.type == PQL_STR_VALUE_B) return (uint32_t)(PQL_OFF_VB + s.owner * 12 + k);
    if (k < 16) return (uint32_t)(PQL_OFF_P0 + s.owner * 16 + k);
    if (k < 32) return (uint32_t)(PQL_OFF_P1 + s.owner * 16 + (k - 16));
    if (s.type == PQL_STR_KEY) {
        if (k < 44) return (uint32_t)(PQL_OFF_P2 + s.owner * 12 + (k - 32));
        return (uint32_t)(PQL_OFF_KP3 + s.owner * 2 + (k - 44));
    }
    return (uint32_t)(PQL_OFF_P2 + s.owner * 8 + (k - 32));
}

/* first byte index after byte k of the string that is not adjacent in the tile to the bytes before it
   (the end of the plane piece that holds byte k) */
PQL_HD int pql_string_run_end(PqString s, int k)
{
    if (s.type == PQL_STR_VALUE_B) return 12;
    if (k < 16) return 16;
    if (k < 32) return 32;
    if (s.type == PQL_STR_KEY) return k < 44 ? 44 : 46;
    return 40;
}

/* Where the fields of block b of slot tau live. */
struct PqBlockPos {
    PqString q_str[2]; /* string holding Q_0, Q_1 / Q_2, Q_3 (keys: the same string twice) */
    int q_bit[4];      /* bit offset of Q_j inside q_str[j >> 1] */
    PqString b_str;
    int b_bit;
    uint32_t radius_half; /* index of the radius inside the tile's 512 halves */
};

PQL_HD PqBlockPos pql_pos(int kind, int tau, int b)
{
    PqBlockPos p;
    if (kind == 0) {
        const PqString s = {PQL_STR_KEY, tau};
        p.q_str[0] = s; p.q_str[1] = s; p.b_str = s;
        for (int j = 0; j < 4; ++j) p.q_bit[j] = PQL_BLOCK_BITS * b + 10 * j;
        p.b_bit = PQL_BLOCK_BITS * b + 40;
        p.radius_half = (uint32_t)(8 * tau + b);
    } else {
        const int i = tau >> 4, g = (tau >> 2) & 3, e = tau & 3, s = 4 * i + e;
        for (int h = 0; h < 2; ++h) {
            const PqString qs = {PQL_STR_VALUE_Q, 16 * g + 2 * b + h};
            p.q_str[h] = qs;
            p.q_bit[2 * h] = PQL_SLOT_BITS * s;
            p.q_bit[2 * h + 1] = PQL_SLOT_BITS * s + 10;
        }
        const PqString bs = {PQL_STR_VALUE_B, 8 * g + b};
        p.b_str = bs;
        p.b_bit = 6 * s;
        p.radius_half = (uint32_t)(16 * (8 * g + b) + s);
    }
    return p;
}

/* `width` (<= 10) bits at bit offset `bit` of a string, read byte by byte (the bytes of a
 * string are not contiguous across its planes). */
PQL_HD uint32_t pql_get_bits(const uint8_t *codes, PqString s, int bit, int width)
{
    const int k = bit >> 3, sh = bit & 7;
    uint32_t v = codes[pql_string_byte(s, k)];
    if (sh + width > 8) v |= (uint32_t)codes[pql_string_byte(s, k + 1)] << 8;
    if (sh + width > 16) v |= (uint32_t)codes[pql_string_byte(s, k + 2)] << 16;
    return (v >> sh) & ((1u << width) - 1u);
}

/* Codes of one block as the levels of the polar transform name them. */
struct PqBlockFields {
    uint32_t l1;      /* 8 level-1 codes, pair p in bits [4p,4p+4) */
    uint32_t g6[2];   /* per half-block h: c2_{2h} << 4 | c3_h << 2 | c2_{2h+1} */
    uint32_t c4;
    uint16_t radius;  /* binary16 bits */
};

/* The stored indices of a block from its codes, and back. */
PQL_HD uint32_t pql_quarter_index(const PqBlockFields &f, int j)
{
    const uint32_t c2 = (j & 1) ? (f.g6[j >> 1] & 3u) : (f.g6[j >> 1] >> 4);
    const uint32_t pairs = (f.l1 >> (8 * j)) & 0xFFu; /* c1_{2j+1} << 4 | c1_{2j} */
    return ((pairs >> 4) << 6) | (c2 << 4) | (pairs & 15u);
}

PQL_HD uint32_t pql_block_index(const PqBlockFields &f)
{
    return (f.c4 << 4) | (((f.g6[0] >> 2) & 3u) << 2) | ((f.g6[1] >> 2) & 3u);
}

PQL_HD PqBlockFields pql_fields_from_indices(const uint32_t (&q)[4], uint32_t bidx, uint16_t radius)
{
    PqBlockFields f;
    f.l1 = 0;
    uint32_t c2[4];
    for (int j = 0; j < 4; ++j) {
        f.l1 |= (((q[j] >> 6) << 4) | (q[j] & 15u)) << (8 * j);
        c2[j] = (q[j] >> 4) & 3u;
    }
    f.g6[0] = (c2[0] << 4) | (((bidx >> 2) & 3u) << 2) | c2[1];
    f.g6[1] = (c2[2] << 4) | ((bidx & 3u) << 2) | c2[3];
    f.c4 = bidx >> 4;
    f.radius = radius;
    return f;
}

/* Generic (slow) reader used by DeQuant and the canonical export.  radii == NULL: the
 * radius field is left zero (caches whose radius plane is not made of block radii). */
PQL_HD PqBlockFields pql_read_block(int kind, const uint8_t *codes, const uint16_t *radii, int tau, int b)
{
    const PqBlockPos p = pql_pos(kind, tau, b);
    uint32_t q[4];
    for (int j = 0; j < 4; ++j) q[j] = pql_get_bits(codes, p.q_str[j >> 1], p.q_bit[j], 10);
    const uint32_t bidx = pql_get_bits(codes, p.b_str, p.b_bit, 6);
    return pql_fields_from_indices(q, bidx, radii ? radii[p.radius_half] : (uint16_t)0);
}

#endif /* PQ_LAYOUT_H */
