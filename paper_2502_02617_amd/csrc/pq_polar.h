/*
 * pq_polar.h -- device code shared by the kernels that encode vectors:
 * procedure Polar with procedure Quant folded in (Algorithm 1) on one block of
 * 16 rotated coordinates, and the decode-time append of one vector.
 */
#ifndef PQ_POLAR_H
#define PQ_POLAR_H

#include "pq_common.h"

#if defined(__HIPCC__)

/* The stored radius is a binary16 number (b_FPN = 16, Section 4.1).  The paper does not say what becomes of a radius
 * beyond that format's range; here it saturates at the largest finite binary16 value, 65504: the block keeps its
 * direction, and everything computed from the cache stays finite. */
__device__ __forceinline__ float pq_saturate_radius(float r) { return fminf(r, 65504.0f); }

/* Quantise one quadrant angle: number of inner boundaries below atan(v/u), for
 * u, v >= 0.  Boundary k is passed when v > t_k * u, that is when the fused
 * t_k * u - v (one rounding, so its sign is the exact one) is negative; the sign
 * bits are added up.  The middle boundary is pi/4 (t = 1). */
__device__ __forceinline__ uint32_t quant3(float u, float v, float t1, float t3)
{
    const float d1 = __builtin_fmaf(t1, u, -v), d2 = u - v, d3 = __builtin_fmaf(t3, u, -v);
    return (__float_as_uint(d1) >> 31) + (__float_as_uint(d2) >> 31) + (__float_as_uint(d3) >> 31);
}

/* First and third inner boundary of each level (the middle one is pi/4): their
 * tangents for level 1, the squares of their tangents above it, where the
 * recursion carries squared radii (v > t u  <=>  v^2 > t^2 u^2 for u, v >= 0). */
struct Thresholds {
    float t1a, t1c, t2a, t2c, t3a, t3c, t4a, t4c;
    float t2b, t3b, t4b; /* middle boundaries (squared tangents), used with general codebooks only */
    float radius_scale;  /* the block radius is multiplied by this (1 unless the rotated coordinates
                            come in scaled; the angles do not depend on a common scale) */
    const PqDeviceConsts::Lut1Cell *lut1; /* level-1 table of general codebooks (LDS or global) */
};

__device__ __forceinline__ Thresholds load_thresholds(const PqDeviceConsts &K, float radius_scale = 1.0f)
{
    Thresholds t;
    t.radius_scale = radius_scale;
    t.lut1 = K.lut1;
    t.t2b = K.tan_b[1][1] * K.tan_b[1][1];
    t.t3b = K.tan_b[2][1] * K.tan_b[2][1];
    t.t4b = K.tan_b[3][1] * K.tan_b[3][1];
    t.t1a = K.tan_b[0][0]; t.t1c = K.tan_b[0][2];
    t.t2a = K.tan_b[1][0] * K.tan_b[1][0]; t.t2c = K.tan_b[1][2] * K.tan_b[1][2];
    t.t3a = K.tan_b[2][0] * K.tan_b[2][0]; t.t3c = K.tan_b[2][2] * K.tan_b[2][2];
    t.t4a = K.tan_b[3][0] * K.tan_b[3][0]; t.t4c = K.tan_b[3][2] * K.tan_b[3][2];
    return t;
}

/* the same with a general middle boundary */
__device__ __forceinline__ uint32_t quant3g(float u, float v, float t1, float t2, float t3)
{
    const float d1 = __builtin_fmaf(t1, u, -v), d2 = __builtin_fmaf(t2, u, -v), d3 = __builtin_fmaf(t3, u, -v);
    return (__float_as_uint(d1) >> 31) + (__float_as_uint(d2) >> 31) + (__float_as_uint(d3) >> 31);
}

/* Level-1 code for general codebooks: pseudo-angle p in [0, 4) of (ya, yb) -- quadrant number plus
 * |yb| / (|ya| + |yb|) in even quadrants, |ya| / (|ya| + |yb|) in odd ones, monotone in the angle --
 * then the cell table: boundaries in earlier cells plus one compare inside the cell. */
__device__ __forceinline__ uint32_t level1_code_general(float ya, float yb, const PqDeviceConsts::Lut1Cell *lut)
{
    const uint32_t ba = __float_as_uint(ya), bb = __float_as_uint(yb);
    const uint32_t sb = bb >> 31, f = (ba ^ bb) >> 31;
    const float a = fabsf(ya), b = fabsf(yb), sum = a + b;
    const float frac = sum > 0.0f ? (f ? a : b) * __builtin_amdgcn_rcpf(sum) : 0.0f;
    const float p = (float)(2u * sb + f) + frac;
    uint32_t cell = (uint32_t)(p * 128.0f);
    cell = cell > 511u ? 511u : cell;
    const PqDeviceConsts::Lut1Cell c = lut[cell];
    return c.count + (p > c.thr ? 1u : 0u);
}

/* What a tile stores of a block (pq_layout.h): the quarter indices Q_j = c1(2j) | c2(j) << 4 | c1(2j+1) << 6 and the
 * block index B = c4 << 4 | c3(0) << 2 | c3(1), put together as the codes come out of the recursion. */
struct BlockCodes {
    uint32_t q[4];
    uint32_t bi;
    uint16_t radius; /* binary16 bits */
    float q4;        /* squared radius of the block (before radius_scale): input of the levels above 4 */
};

/* Levels 5, 6, 7 of a vector from the squared radii of its blocks (full-depth recursion):
 * lo = blocks 0..3, hi = blocks 4..7.  Returns the radius-plane word of the vector:
 * binary16 radius << 16 | codes (level-5 codes j = 0..3 at bits [j b5, (j+1) b5), level 6
 * above them, level 7 on top). */
struct UpperHalf {
    uint32_t codes; /* this half's level-5 and level-6 codes, already at their bit positions */
    float q6;       /* squared radius of the half */
};

/* boundaries and widths of levels 5..7, read once per kernel (the same in all lanes) */
struct UpperTables {
    float tan2[3][7];
    int b5, b6, b7;
};

__device__ __forceinline__ UpperTables load_upper_tables(const PqDeviceConsts &K)
{
    UpperTables u;
#pragma unroll
    for (int l = 0; l < 3; ++l)
#pragma unroll
        for (int k = 0; k < 7; ++k) u.tan2[l][k] = K.up_tan2[l][k];
    u.b5 = K.up_bits[0]; u.b6 = K.up_bits[1]; u.b7 = K.up_bits[2];
    return u;
}

__device__ __forceinline__ UpperHalf polar_upper_half(const float (&q4)[4], int half, const UpperTables &K)
{
    const uint32_t c5a = pq_quant_upper(q4[0], q4[1], K.tan2[0], (1 << K.b5) - 1);
    const uint32_t c5b = pq_quant_upper(q4[2], q4[3], K.tan2[0], (1 << K.b5) - 1);
    const float q5a = q4[0] + q4[1], q5b = q4[2] + q4[3];
    const uint32_t c6 = pq_quant_upper(q5a, q5b, K.tan2[1], (1 << K.b6) - 1);
    UpperHalf h;
    h.codes = ((c5a | (c5b << K.b5)) << (2 * K.b5 * half)) | (c6 << (4 * K.b5 + K.b6 * half));
    h.q6 = q5a + q5b;
    return h;
}

__device__ __forceinline__ uint32_t polar_upper_join(const UpperHalf &lo, const UpperHalf &hi, float radius_scale,
                                                     const UpperTables &K)
{
    const uint32_t c7 = pq_quant_upper(lo.q6, hi.q6, K.tan2[2], (1 << K.b7) - 1);
    const float r7 = pq_saturate_radius(__builtin_amdgcn_sqrtf(lo.q6 + hi.q6) * radius_scale);
    const _Float16 rh = (_Float16)r7; /* round to nearest even */
    return lo.codes | hi.codes | (c7 << (4 * K.b5 + 2 * K.b6)) | ((uint32_t)__builtin_bit_cast(uint16_t, rh) << 16);
}

/* Procedure Polar on one block of 16 rotated coordinates with procedure Quant
 * folded in: four levels of (angle code, radius) pairs, all in registers.  Only
 * the squares of the intermediate radii are kept (the angle of a node depends on
 * the ratio of its children's radii alone); the root radius takes the one square
 * root.  The recursion is cut into eight steps (one level-1 pair each, plus the
 * nodes of the upper levels that the pair completes) so that a caller can spread
 * it between other work. */
struct PolarState {
    float q1[8], q2[4], q3[2]; /* squared radii */
    uint32_t mq, c3[2];
    BlockCodes out;
};

/* level-1 pair p, first part: position inside the quadrant */
template <bool GENERAL = false, typename Y16>
__device__ __forceinline__ void polar_level1_a(PolarState &s, const Y16 &y, int p, const Thresholds &th)
{
    if (GENERAL) s.mq = level1_code_general(y[2 * p], y[2 * p + 1], th.lut1); /* the whole code */
    else s.mq = quant3(fabsf(y[2 * p]), fabsf(y[2 * p + 1]), th.t1a, th.t1c);
}

/* level-1 pair p, second part: quadrant, code, squared radius */
template <bool GENERAL = false, typename Y16>
__device__ __forceinline__ void polar_level1_b(PolarState &s, const Y16 &y, int p)
{
    const float ya = y[2 * p], yb = y[2 * p + 1];
    uint32_t code;
    if (GENERAL) {
        code = s.mq;
    } else {
        /* cell of atan2(yb, ya) in [0, 2 pi), cells pi/8 wide: quadrant Q = 0..3 from the signs,
           code = 4Q + mq in quadrants 0 and 2, 4Q + 3 - mq in 1 and 3 (angle measured from the
           other axis), which is (mq xor 7f) | 8 sb with f = sa xor sb */
        const uint32_t ba = __float_as_uint(ya), bb = __float_as_uint(yb);
        const uint32_t f7 = (uint32_t)((int32_t)(ba ^ bb) >> 31) & 7u;
        code = (s.mq ^ f7) | ((bb >> 28) & 8u); /* the first term is below 8 */
    }
    s.out.q[p >> 1] = (p & 1) ? (s.out.q[p >> 1] | (code << 6)) : code;
    s.q1[p] = __builtin_fmaf(ya, ya, yb * yb);
}

/* the upper-level nodes whose children are complete once level-1 pair p is done */
template <bool GENERAL = false>
__device__ __forceinline__ void polar_upper(PolarState &s, int p, const Thresholds &th)
{
    if (p & 1) {
        const int n = p >> 1;
        const uint32_t c2 = GENERAL ? quant3g(s.q1[2 * n], s.q1[2 * n + 1], th.t2a, th.t2b, th.t2c)
                                    : quant3(s.q1[2 * n], s.q1[2 * n + 1], th.t2a, th.t2c);
        s.out.q[n] |= c2 << 4;
        s.q2[n] = s.q1[2 * n] + s.q1[2 * n + 1];
    }
    if ((p & 3) == 3) {
        const int h = p >> 2;
        s.c3[h] = GENERAL ? quant3g(s.q2[2 * h], s.q2[2 * h + 1], th.t3a, th.t3b, th.t3c)
                          : quant3(s.q2[2 * h], s.q2[2 * h + 1], th.t3a, th.t3c);
        s.q3[h] = s.q2[2 * h] + s.q2[2 * h + 1];
    }
    if (p == 7) {
        const uint32_t c4 = GENERAL ? quant3g(s.q3[0], s.q3[1], th.t4a, th.t4b, th.t4c)
                                    : quant3(s.q3[0], s.q3[1], th.t4a, th.t4c);
        s.out.bi = (c4 << 4) | (s.c3[0] << 2) | s.c3[1];
        s.out.q4 = s.q3[0] + s.q3[1];
        const float r4 = pq_saturate_radius(__builtin_amdgcn_sqrtf(s.out.q4) * th.radius_scale);
        const _Float16 rh = (_Float16)r4; /* round to nearest even */
        s.out.radius = __builtin_bit_cast(uint16_t, rh);
    }
}

template <bool GENERAL = false, typename Y16>
__device__ __forceinline__ BlockCodes polar_quant_block(const Y16 &y, const Thresholds &th)
{
    PolarState s;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        polar_level1_a<GENERAL>(s, y, p, th);
        polar_level1_b<GENERAL>(s, y, p);
        polar_upper<GENERAL>(s, p, th);
    }
    return s.out;
}

/* ---- decode-time append: one vector per (sequence, head) ----
 * Too little work for the matrix cores: one workgroup per vector computes
 * y_j = sum_i x_i S[i][j] in fp32 (S read from L2, four partial sums per
 * coordinate added in a fixed order), the first wavefront then runs the polar recursion
 * (one lane per level-1 pair) and patches the fields into the tile in place.  Fields share dwords with other
 * slots of the tile, so they are updated with dword atomics. */
struct AppendArgs {
    const void *x;
    uint8_t *codes;
    uint16_t *radii;
    int64_t pool_tiles, pool_tokens;
    const int64_t *dst_token;
    int n_heads;
    const float *S; /* S[i*128 + j] */
    const PqDeviceConsts *consts;
    PqHadamard had; /* on: y = x S by a fast Walsh-Hadamard transform, S is not read */
};

/* Sets `width` (<= 32) bits at bit offset `bit` of a layout string inside a tile's code bytes (global memory
 * or an LDS image of the tile) to v.  Inside a plane the bytes of a string are contiguous, so a run of bits goes
 * in with one update of the dword pair that holds it; a run ends where the string moves on to its next plane.
 * Other lanes update neighbouring fields of the same dwords at the same time: dword atomics.
 * CLEAR = false: the bits are known to be zero. */
template <bool CLEAR>
__device__ __forceinline__ void pql_put_bits(uint32_t *tile_dwords, PqString s, int bit, int width, uint32_t v)
{
    while (width > 0) {
        const int k = bit >> 3;
        const int run = min(width, 8 * pql_string_run_end(s, k) - bit); /* bits that are contiguous in the tile */
        const uint32_t at_bit = 8u * pql_string_byte(s, k) + (uint32_t)(bit & 7);
        const uint32_t dw = at_bit >> 5, sh = at_bit & 31u;
        const uint64_t mask = (run >= 32 ? 0xFFFFFFFFull : ((1ull << run) - 1ull)) << sh;
        const uint64_t val = ((uint64_t)v << sh) & mask;
        if (CLEAR) atomicAnd(&tile_dwords[dw], ~(uint32_t)mask);
        atomicOr(&tile_dwords[dw], (uint32_t)val);
        if (mask >> 32) {
            if (CLEAR) atomicAnd(&tile_dwords[dw + 1], ~(uint32_t)(mask >> 32));
            atomicOr(&tile_dwords[dw + 1], (uint32_t)(val >> 32));
        }
        v = run >= 32 ? 0u : v >> run;
        bit += run;
        width -= run;
    }
}

/* all code fields of block b of slot tau (not the radius) */
template <bool CLEAR>
__device__ __forceinline__ void pql_put_block(uint32_t *tile_dwords, int kind, int tau, int b, const PqBlockFields &f)
{
    const PqBlockPos pos = pql_pos(kind, tau, b);
    const uint32_t q0 = pql_quarter_index(f, 0), q1 = pql_quarter_index(f, 1), q2 = pql_quarter_index(f, 2),
                   q3 = pql_quarter_index(f, 3), bi = pql_block_index(f);
    if (kind == 0) { /* one run of 46 bits: Q_0 | Q_1 << 10 | Q_2 << 20 | Q_3 << 30 | B << 40 */
        pql_put_bits<CLEAR>(tile_dwords, pos.b_str, pos.q_bit[0], 32, q0 | (q1 << 10) | (q2 << 20) | (q3 << 30));
        pql_put_bits<CLEAR>(tile_dwords, pos.b_str, pos.q_bit[0] + 32, 14, (q3 >> 2) | (bi << 8));
    } else {  /* two slots of 20 bits and the block index */
        pql_put_bits<CLEAR>(tile_dwords, pos.q_str[0], pos.q_bit[0], 20, q0 | (q1 << 10));
        pql_put_bits<CLEAR>(tile_dwords, pos.q_str[1], pos.q_bit[2], 20, q2 | (q3 << 10));
        pql_put_bits<CLEAR>(tile_dwords, pos.b_str, pos.b_bit, 6, bi);
    }
}

/* one (sequence, head) vector of kind `kind`, by one workgroup */
template <int XT>
__device__ __forceinline__ void append_vector(const AppendArgs &a, int kind, int vec)
{
    __shared__ float sx[PQ_D];
    __shared__ float sy[PQ_D];
    __shared__ float spart[4][PQ_D];
    const int seq = vec / a.n_heads, head = vec % a.n_heads, tid = threadIdx.x, j = tid & 127;
    MatrixSlice ms;
    if (!a.had.on) matrix_slice_load(ms, a.S, tid);
    const int64_t dst = a.dst_token[seq];
    if (dst < 0 || dst >= a.pool_tokens) return; /* slot outside the pool: nothing is written */
    const int64_t row = ((int64_t)seq * a.n_heads + head) * PQ_D;
    if (tid < PQ_D) {
        if (XT == PQ_BF16) sx[j] = __uint_as_float((uint32_t)static_cast<const uint16_t *>(a.x)[row + j] << 16);
        else sx[j] = static_cast<const float *>(a.x)[row + j];
    }
    __syncthreads();
    /* y_j = sum_i x_i S[i][j].  Hadamard S: the transform of D x, left unscaled -- the angles do not see the
       common factor 1/sqrt(128), which goes into the radius (as in the encode kernel's one-term product) */
    float radius_scale = 1.0f;
    if (a.had.on) {
        if (tid < 64) {
            float lo = sx[tid] * pq_hadamard_sign(a.had, tid), hi = sx[tid + 64] * pq_hadamard_sign(a.had, tid + 64);
            pq_fwht128(lo, hi, tid);
            sy[tid] = lo;
            sy[tid + 64] = hi;
        }
        radius_scale = PQ_INV_SQRT_D;
    } else {
        const float acc = vector_times_slice(sx, ms, spart, tid);
        if (tid < PQ_D) sy[j] = acc;
    }
    __syncthreads();
    __shared__ float sq4[8];
    const bool deep = a.consts->depth == 7;
    const int64_t tile = dst >> 6;
    const int tau = (int)(dst & 63);
    if (tid < 64) {
        /* The first wavefront runs the recursion with one lane per level-1 pair: lane p holds pair p & 7
           of block p >> 3; the nodes of the upper levels sit in the lanes of their first leaf and fetch
           the sibling's squared radius with a shuffle (the other lanes compute along and are ignored).
           Operations and operand order per node are those of polar_quant_block. */
        const int p = tid, i = p & 7, b = p >> 3;
        const Thresholds th = load_thresholds(*a.consts, radius_scale);
        const float ya = sy[2 * p], yb = sy[2 * p + 1];
        uint32_t code1;
        if (a.consts->general) { /* the level-1 table is read from the constants in global memory */
            code1 = level1_code_general(ya, yb, th.lut1);
        } else {
            const uint32_t mq = quant3(fabsf(ya), fabsf(yb), th.t1a, th.t1c);
            const uint32_t ba = __float_as_uint(ya), bb = __float_as_uint(yb);
            const uint32_t f7 = (uint32_t)((int32_t)(ba ^ bb) >> 31) & 7u;
            code1 = (mq ^ f7) | ((bb >> 28) & 8u);
        }
        const float q1 = __builtin_fmaf(ya, ya, yb * yb);
        const float q1s = __shfl_xor(q1, 1);
        const uint32_t c2 = a.consts->general ? quant3g(q1, q1s, th.t2a, th.t2b, th.t2c) : quant3(q1, q1s, th.t2a, th.t2c);
        const float q2 = q1 + q1s;
        const float q2s = __shfl_xor(q2, 2);
        const uint32_t c3 = a.consts->general ? quant3g(q2, q2s, th.t3a, th.t3b, th.t3c) : quant3(q2, q2s, th.t3a, th.t3c);
        const float q3 = q2 + q2s;
        const float q3s = __shfl_xor(q3, 4);
        PqBlockFields bc;
        bc.c4 = a.consts->general ? quant3g(q3, q3s, th.t4a, th.t4b, th.t4c) : quant3(q3, q3s, th.t4a, th.t4c);
        const float q4 = q3 + q3s;
        const _Float16 rh = (_Float16)pq_saturate_radius(__builtin_amdgcn_sqrtf(q4) * th.radius_scale); /* round to nearest even */
        bc.radius = __builtin_bit_cast(uint16_t, rh);
        /* the block's fields gathered into its first lane: level-1 codes at their nibbles; the 6-bit
           groups [c2(2h) | c3(h) | c2(2h+1)] of half-block h at bits [8h, 8h+6) of a second word */
        uint32_t l1 = code1 << (4 * i);
        uint32_t gw = (i & 1) ? 0u : ((i & 2) ? c2 : ((c2 << 4) | (c3 << 2))) << (2 * (i & 4));
#pragma unroll
        for (int d = 1; d < 8; d <<= 1) {
            l1 |= __shfl_xor(l1, d);
            gw |= __shfl_xor(gw, d);
        }
        bc.l1 = l1;
        bc.g6[0] = gw & 63u;
        bc.g6[1] = (gw >> 8) & 63u;
        if (i == 0) {
            uint8_t *gcodes = a.codes + ((int64_t)head * a.pool_tiles + tile) * PQL_CODE_BYTES;
            pql_put_block<true>(reinterpret_cast<uint32_t *>(gcodes), kind, tau, b, bc);
            if (deep) sq4[b] = q4;
            else a.radii[((int64_t)head * a.pool_tiles + tile) * PQL_RADII + pql_pos(kind, tau, b).radius_half] = bc.radius;
        }
    }
    if (deep) { /* levels 5..7 over the eight block radii: one thread, one whole word of the radius plane */
        __syncthreads();
        if (tid == 0) {
            const float lo4[4] = {sq4[0], sq4[1], sq4[2], sq4[3]}, hi4[4] = {sq4[4], sq4[5], sq4[6], sq4[7]};
            const UpperTables ut = load_upper_tables(*a.consts);
            const UpperHalf lo = polar_upper_half(lo4, 0, ut), hi = polar_upper_half(hi4, 1, ut);
            uint32_t *top = reinterpret_cast<uint32_t *>(a.radii) +
                            ((int64_t)head * a.pool_tiles + tile) * (PQ_DEEP_RADII_HALVES / 2);
            top[tau] = polar_upper_join(lo, hi, radius_scale, ut);
        }
    }
}

#endif /* __HIPCC__ */
#endif /* PQ_POLAR_H */
