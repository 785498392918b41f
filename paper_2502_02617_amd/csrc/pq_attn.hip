/*
 * pq_attn.hip -- pq_attn_decode_polar and its relatives (the whole decode step,
 * several query tokens per sequence, a quantised prefix plus an unquantised
 * window): attention computed directly on the packed PolarQuant cache (Eq. 5
 * with the DeQuant of Algorithm 1 fused in), for gfx950.
 *
 * Because S is a rotation, <q, khat> = <q S, khat S>: keys and values stay in
 * the rotated domain r^(0) (DeQuant without its trailing S^T), the query is
 * rotated once and the weighted value sum is multiplied by S^T once.
 *
 * Three kernels per call:
 *   pq_rotate_q_kernel      q' = (q S) * softmax_scale * log2(e), binary16; one more
 *                           workgroup builds the work plan from ctx_len: an equal
 *                           share of all tiles for every wavefront of the next launch
 *   pq_attn_partial_kernel  one wavefront per share: streams the K and V tiles of
 *                           its piece(s) of (sequence, kv head) streams, rebuilds
 *                           them in registers, scores and weighted sums on the matrix
 *                           cores, online softmax; writes (m, l, o') per piece
 *   pq_attn_combine_kernel  merges the pieces of a (sequence, query head) in tile
 *                           order, divides by l, multiplies by S^T, bf16
 *
 * Partial kernel, per 64-token tile (the cache stores, per block of 16 coordinates, four 10-bit quarter
 * indices Q, one 6-bit block index B and the binary16 block radius: pq_layout.h):
 *   K:  one token per lane.  For each of the token's 32 quarters the lane fetches the quarter's table
 *       entry -- the four binary16 products (cos|sin) theta2 * (cos|sin) theta1 -- and hands it to
 *       v_mfma_f32_4x4x4_16b_f16 as it is: the matrix cores form the 4-coordinate inner products with
 *       q' for four (query token, head) pairs.  Each result is multiplied in fp32 by the quarter's
 *       radius (block radius x block-table entry (cos|sin) theta4 * (cos|sin) theta3) and added to the
 *       token's scores.  At recursion depth 7 the lane first rebuilds its token's block radii from the
 *       vector's radius and its upper-level codes.
 *   softmax: probabilities 2^(s - m + 9) against a lagging exponent reference m per pair; a lane holds
 *       the four pairs of its token, and hands them through LDS to the lanes that need them as operands.
 *   V:  four passes of 16 tokens.  Lane (g, n) rebuilds half-block n (8 coordinates) of tokens
 *       16 i + 4 g + {0..3} with packed binary16 multiplies: radius x block-table entry -> the radii of
 *       the half's two quarters, times the two quarter entries.  A register of a quarter entry holds two
 *       coordinates of one token, while a matrix-core operand wants several tokens of one coordinate per
 *       lane; instead of transposing, the contraction index of v_mfma_f32_16x16x32_f16 is widened to
 *       (token, parity): operand rows are coordinate pairs, and the probability operand has one column per
 *       (pair, parity) with zeros in the slots of the other parity.  The result accumulates o' for the
 *       even coordinates in the parity-0 columns and for the odd ones in parity 1.
 */
#include <type_traits>

#include "pq_common.h"
#include "pq_polar.h"

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));

/* One workgroup per CU: the lookup tables are laid out in LDS with a private bank column per lane (see
 * stage_tables), which takes 48 KB, so all wavefronts resident on a CU share one copy: 4 SIMDs x the
 * wavefronts per SIMD that the variant's register budget allows. */
constexpr int waves_per_simd(int NG) { return NG == 1 ? 4 : (NG == 2 ? 3 : 2); }
constexpr int waves_per_block(int NG) { return 4 * waves_per_simd(NG); }
constexpr float kLog2e = 1.4426950408889634f;
/* Probabilities are handed to the matrix cores as binary16.  They are computed
 * as 2^(s - m + kProbShift) against an exponent reference m that may lag the true
 * maximum by up to kRefSlack, so that weights from 2^-23 below the reference (normal
 * numbers) to 2^kRefSlack above it fit; l carries the same factor and it cancels in o'/l. */
constexpr float kProbShift = 9.0f;
constexpr float kRefSlack = 6.0f;

/* LDS table block: layout in pq_common.h (PQ_TAB_*), image built on the host */
constexpr int kTabDwords = PQ_TAB_DWORDS;
/* The tables as the kernel lays them out in LDS (dwords).  Random gathers from a table collide in the LDS banks
 * unless every lane that is served in the same cycle reads its own bank: a 4-byte gather is served 32 lanes at a
 * time, a 16-byte gather 16 lanes at a time, so the small tables are replicated into one column per lane (mod 32,
 * mod 16) -- entry e of lane l at row e, column l -- and their gathers never collide (2.4 instead of 4.1 cycles
 * per 4-byte gather from 64 entries, 4.6 instead of 10.4 per 16-byte gather).
 *   kTQ   [1024][2]       quarter table, by Q (8 KB, gathered as it is: 32 columns of it would be 256 KB)
 *   kTQA  [64][32]        first pair of a quarter, by Q & 63 = c2 << 4 | c1
 *   kTQB  [64][32]        second pair, by Q >> 4 = c1' << 2 | c2
 *   kTBF  [64][16][4]     block table of the keys (fp32), by B
 *   kTBH  [64][32]        block table of the values: column l holds the binary16 pair of half-block l & 1
 *   kTUp  [3][8][2]       levels 5..7 (full depth) */
constexpr int kTQ = 0, kTQA = 2048, kTQB = 4096, kTBF = 6144, kTBH = 10240, kTUp = 12288, kLdsTabDwords = 12336;
/* how a quarter's table entry is fetched: as one 8-byte gather from kTQ (bank conflicts, but one index), or as
   two conflict-free 4-byte gathers from the pair tables (two indices) */
#ifndef PQ_KEY_PAIRS
#define PQ_KEY_PAIRS 1
#endif
#ifndef PQ_VALUE_PAIRS
#define PQ_VALUE_PAIRS 0
#endif

struct AttnArgs {
    const uint16_t *qrot; /* [B][M][Hq][128] binary16: rotated, pre-scaled q' */
    const uint8_t *k_codes, *v_codes;
    const uint16_t *k_radii, *v_radii;
    int up_b5, up_b6, up_b7; /* bits of levels 5, 6, 7 (depth 7 only) */
    const int64_t *seq_start;
    const int32_t *ctx_len;
    int B, Hq, Hkv;
    int M; /* query tokens per sequence: rows are ordered [B][M][Hq] */
    int64_t pool_tiles;
    int64_t max_ctx;
    const int32_t *plan; /* device work plan, see below */
    int n_pieces;        /* piece ids run below this (sizes ws_ml, ws_o) */
    float *ws_ml; /* [piece][M * G pairs][2] */
    float *ws_o;  /* [piece][M * G pairs][128] */
    const PqDeviceConsts *consts;
};

/* Work plan of one attention call, built on the device from ctx_len by the launch that
 * precedes the partial kernel (the host never reads the context lengths).  The tiles of all
 * (sequence, kv head) streams form one global sequence, stream (b, hk) before (b, hk + 1)
 * before (b + 1, 0); wavefront w of the partial kernel takes global tiles
 * [w * share, (w + 1) * share): every wavefront gets the same number of tiles whatever
 * the mix of context lengths, and a wavefront whose range crosses a stream boundary works
 * through one piece per stream.  Piece ids are w + (b * Hkv + hk): along the global
 * sequence either w or the stream index grows from one piece to the next, so the id is unique
 * and the pieces of one stream are consecutive ids.
 * All counts fit 31 bits (the launch code refuses batches whose tile count could not).
 *   plan[0] = total tiles (all streams), plan[1] = share (tiles per wavefront),
 *   plan[2 + b] = tiles of sequences 0 .. b-1 of ONE kv head (b = 0 .. B), then for every
 *   stream s = b * Hkv + hk, from plan[2 + B + 1 + 2 s]: the wavefront of its first piece and
 *   the number of its pieces (what the combine kernel needs). */
constexpr int kPlanHeader = 2;
constexpr int kMinShareTiles = 4;

typedef _Float16 h4 __attribute__((ext_vector_type(4)));

union H8 {
    h8 v;
    uint4 q;
    uint32_t w[4];
    h2 p[4];
};

union H4 {
    h4 v;
    uint2 d;
    uint32_t w[2];
    h2 p[2];
};

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 v) { return __builtin_bit_cast(uint32_t, v); }

__device__ __forceinline__ h2 bcast_lo(h2 v) { return h2{v.x, v.x}; }
__device__ __forceinline__ h2 bcast_hi(h2 v) { return h2{v.y, v.y}; }

/* A 32-bit literal doubles the size of a vector instruction; masks used hundreds of times
 * per tile are kept in scalar registers instead (the empty asm hides their value from
 * constant propagation). */
__device__ __forceinline__ uint32_t scalar_const(uint32_t v)
{
    asm("" : "+s"(v));
    return v;
}

/* Byte offset of a table entry from the index stored at bit BIT of the little-endian bit string
 * w[0], w[1], ...: (index << SHIFT), entries of 2^SHIFT bytes.  The position is a compile-time
 * constant, so this is one shift (a funnel shift where the field straddles two dwords) and one
 * mask-and-or; a field that already sits at bit SHIFT of its dword needs the latter only. */
template <int BIT, int WIDTH, int SHIFT>
__device__ __forceinline__ uint32_t table_offset(const uint32_t *w, uint32_t column = 0u)
{
    constexpr int d = BIT >> 5, s = BIT & 31;
    const uint32_t mask = scalar_const(((1u << WIDTH) - 1u) << SHIFT);
    uint32_t v;
    if constexpr (s + WIDTH <= 32) {
        if constexpr (s == SHIFT) v = w[d];
        else if constexpr (s > SHIFT) v = w[d] >> (s - SHIFT);
        else v = w[d] << (SHIFT - s);
    } else {
        static_assert(s + WIDTH <= 32 || s >= SHIFT, "a straddling field starts above bit SHIFT");
        v = __builtin_amdgcn_alignbit(w[d + 1], w[d], s - SHIFT);
    }
    return (v & mask) | column; /* column: the lane's byte offset inside a row of a table with a column per lane */
}

/* The four binary16 values of a quarter from the 10-bit index stored at bit BIT of the string w: either entry Q of
 * the quarter table, or entries Q & 63 and Q >> 4 of the two pair tables (col4 = 4 * (lane & 31)). */
template <int BIT, bool PAIRS>
__device__ __forceinline__ uint2 quarter_entry(const uint32_t *tab, const uint32_t *w, uint32_t col4)
{
    if constexpr (PAIRS) {
        const uint32_t oa = table_offset<BIT, 6, 7>(w, col4), ob = table_offset<BIT + 4, 6, 7>(w, col4);
        return make_uint2(*reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(tab + kTQA) + oa),
                          *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(tab + kTQB) + ob));
    } else {
        const uint32_t o = table_offset<BIT, 10, 3>(w);
        return *reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(tab + kTQ) + o);
    }
}

/* Raw registers of a key tile: lane tau holds token tau -- its 46 code bytes (12 dwords, the last one
 * half used) and its 8 block radii, or at depth 7 its word of the radius plane. */
struct KTileRaw {
    uint32_t w[12];
    uint4 rad;
    uint32_t top;
};

/* Raw registers of a value tile: lane (g, n) holds the 40-byte index string of half-block n for its 16
 * token slots, the 12-byte block-index string and the 16 radii of its block (both shared with the lane
 * of the block's other half), or at depth 7 the radius-plane word of token `lane`. */
struct VTileRaw {
    uint32_t q[10];
    uint32_t b[3];
    uint4 rad0, rad1; /* slots 0..7 | 8..15 */
    uint32_t top;
};

/* The tiles of one (sequence, kv head) stream are read through buffer descriptors: the address of a
 * field is (descriptor base, scalar tile offset, 32-bit lane offset), so no 64-bit per-lane address
 * registers are carried through the tile loop.  The kernel only forms offsets of tiles below the
 * sequence's tile count, which is also the size the descriptor is given. */
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t stream_descriptor(const void *base, uint32_t bytes)
{
    /* raw buffer (stride 0), 32-bit data format word as for every untyped dword access on this family */
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint4 load16(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t tile_off)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, tile_off, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

/* The lane offsets are recomputed for every tile from the lane number (a handful of shifts), which the
 * empty asm statement hides from loop-invariant code motion: hoisted, they would cost more registers
 * than the kernel has and come back as spills inside the tile loop.  Plane offsets ride on the scalar
 * tile offset. */
template <bool DEEP>
__device__ __forceinline__ void load_k_tile(KTileRaw &t, __amdgpu_buffer_rsrc_t codes, __amdgpu_buffer_rsrc_t radii,
                                            uint32_t tile, uint32_t lane)
{
    asm volatile("" : "+v"(lane));
    const uint32_t co = tile * PQL_CODE_BYTES;
    const uint4 a = load16(codes, lane * 16u, co + PQL_OFF_P0);
    const uint4 b = load16(codes, lane * 16u, co + PQL_OFF_P1);
    const u32x3 c = __builtin_amdgcn_raw_buffer_load_b96(codes, lane * 12u, co + PQL_OFF_P2, 0);
    t.w[0] = a.x; t.w[1] = a.y; t.w[2] = a.z; t.w[3] = a.w;
    t.w[4] = b.x; t.w[5] = b.y; t.w[6] = b.z; t.w[7] = b.w;
    t.w[8] = c.x; t.w[9] = c.y; t.w[10] = c.z;
    t.w[11] = __builtin_amdgcn_raw_buffer_load_b16(codes, lane * 2u, co + PQL_OFF_KP3, 0);
    if (DEEP) t.top = __builtin_amdgcn_raw_buffer_load_b32(radii, lane * 4u, tile * (PQ_DEEP_RADII_HALVES * 2u), 0);
    else t.rad = load16(radii, lane * 16u, tile * (PQL_RADII * 2u));
}

template <bool DEEP>
__device__ __forceinline__ void load_v_tile(VTileRaw &t, __amdgpu_buffer_rsrc_t codes, __amdgpu_buffer_rsrc_t radii,
                                            uint32_t tile, uint32_t lane)
{
    asm volatile("" : "+v"(lane));
    const uint32_t co = tile * PQL_CODE_BYTES;
    const uint4 a = load16(codes, lane * 16u, co + PQL_OFF_P0);
    const uint4 b = load16(codes, lane * 16u, co + PQL_OFF_P1);
    const u32x2 c = __builtin_amdgcn_raw_buffer_load_b64(codes, lane * 8u, co + PQL_OFF_P2, 0);
    const u32x3 x = __builtin_amdgcn_raw_buffer_load_b96(codes, (lane >> 1) * 12u, co + PQL_OFF_VB, 0);
    t.q[0] = a.x; t.q[1] = a.y; t.q[2] = a.z; t.q[3] = a.w;
    t.q[4] = b.x; t.q[5] = b.y; t.q[6] = b.z; t.q[7] = b.w;
    t.q[8] = c.x; t.q[9] = c.y;
    t.b[0] = x.x; t.b[1] = x.y; t.b[2] = x.z;
    if (DEEP) {
        t.top = __builtin_amdgcn_raw_buffer_load_b32(radii, lane * 4u, tile * (PQ_DEEP_RADII_HALVES * 2u), 0);
    } else {
        t.rad0 = load16(radii, (lane >> 1) * 32u, tile * (PQL_RADII * 2u));
        t.rad1 = load16(radii, (lane >> 1) * 32u, tile * (PQL_RADII * 2u) + 16u);
    }
}

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

/* Depth 7: the block radii of a tile are not stored but rebuilt from each token's radius and its
 * codes of levels 7, 6, 5 (DeQuant's first three steps).  On the key side lane tau does that for its
 * own token, in registers.  On the value side lane tau does it for token tau and leaves the eight radii
 * in LDS as binary16 in the order in which the passes read the stored radii of a depth-4 tile:
 * vrad[(8 g + b) * 16 + 4 i + e] = radius of block b of token 16 i + 4 g + e. */
struct DeepRadii {
    uint16_t *vrad;    /* [512] */
    int b5, b6, b7;
};

__device__ __forceinline__ void stage_deep_value_radii(const uint32_t *tab, const DeepRadii &dr, uint32_t vtop, int lane)
{
    const float2 *cs = reinterpret_cast<const float2 *>(tab + kTUp);
    float r[8];
    pq_deep_block_radii(vtop, dr.b5, dr.b6, dr.b7, cs, r);
    const int i = lane >> 4, g = (lane >> 2) & 3, e = lane & 3;
#pragma unroll
    for (int b = 0; b < 8; ++b)
        dr.vrad[(8 * g + b) * 16 + 4 * i + e] = __builtin_bit_cast(uint16_t, (_Float16)r[b]);
}

/* Context length the kernels act on: the caller's value clamped to [0, max_ctx];
 * a sequence whose slots would leave the pool or that does not start on a tile
 * boundary is treated as empty (zero output) instead of being read. */
__device__ __forceinline__ int effective_ctx_of(int64_t c, int64_t s0, int64_t max_ctx, int64_t pool_tiles)
{
    if (c > max_ctx) c = max_ctx;
    if (c <= 0) return 0;
    if (s0 < 0 || (s0 & 63) || (s0 >> 6) + ((c + 63) >> 6) > pool_tiles) return 0;
    return (int)c;
}

__device__ __forceinline__ int effective_ctx(const int64_t *seq_start, const int32_t *ctx_len, int b,
                                             int64_t max_ctx, int64_t pool_tiles)
{
    return effective_ctx_of(ctx_len[b], seq_start[b], max_ctx, pool_tiles); /* two independent loads */
}

/* Issue priority of the wavefront among those of its SIMD (0..3, scalar argument). */
__device__ __forceinline__ void set_wave_priority(int prio)
{
    if (prio <= 0) __builtin_amdgcn_s_setprio(0);
    else if (prio == 1) __builtin_amdgcn_s_setprio(1);
    else if (prio == 2) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(3);
}

__device__ __forceinline__ uint32_t sel4(uint4 v, int c)
{
    return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w));
}

__device__ __forceinline__ float half_lo_to_float(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xFFFFu)); }
__device__ __forceinline__ float half_hi_to_float(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); }

/* Query operand of the scores: for column group k, a[k][set] holds in lane (i = lane >> 2, slot = lane & 3) the four
 * rotated query coordinates 4 x .. 4 x + 3 of quarter x = 16 set + i for pair 4 k + slot, in binary16.
 * v_mfma_f32_4x4x4_16b_f16 multiplies 16 independent 4x4 blocks; with the A block of one lane group broadcast to
 * all sixteen (cbsz = 4, abid = i) one register pair serves sixteen quarters. */
template <int NG> struct QueryOperand { H4 a[NG][2]; };

/* Scores of one 64-token tile, one token per lane (Eq. 5 with DeQuant unrolled into table products):
 *   s_pair(tau) = sum_b r_b(tau) sum_j T43[B_b][j] * < q'[16 b + 4 j .. + 3], T21[Q_{b,j}] >
 * T21[Q] (binary16, from LDS) = the four products (cos|sin) theta2 * (cos|sin) theta1 of a quarter -- it is the B
 * operand of the matrix instruction as fetched; T43[B] (fp32) = the four products (cos|sin) theta4 * (cos|sin)
 * theta3 of a block.  The matrix cores form the 4-coordinate inner products of a quarter for four (query token,
 * head) pairs per group; each is scaled in fp32
 * by r_b T43[B_b][j] and summed.  A key element is therefore never rounded beyond its table entry.
 * s comes in holding the negated exponent reference (the first product of a tile adds to it). */
template <int NG, bool DEEP>
__device__ __forceinline__ void key_scores(const uint32_t *tab, const KTileRaw &k, const QueryOperand<NG> &qo,
                                           float (&s)[NG][4], const DeepRadii &dr, int lane)
{
    const f4 zero = f4{0.f, 0.f, 0.f, 0.f};
    float rb[8];
    if (DEEP) {
        pq_deep_block_radii(k.top, dr.b5, dr.b6, dr.b7, reinterpret_cast<const float2 *>(tab + kTUp), rb);
    } else {
        rb[0] = half_lo_to_float(k.rad.x); rb[1] = half_hi_to_float(k.rad.x);
        rb[2] = half_lo_to_float(k.rad.y); rb[3] = half_hi_to_float(k.rad.y);
        rb[4] = half_lo_to_float(k.rad.z); rb[5] = half_hi_to_float(k.rad.z);
        rb[6] = half_lo_to_float(k.rad.w); rb[7] = half_hi_to_float(k.rad.w);
    }
    const uint32_t col4 = (uint32_t)(lane & 31) * 4u, col16 = (uint32_t)(lane & 15) * 16u;
    auto block = [&](auto bc) {
        constexpr int b = decltype(bc)::value;
        const uint32_t boff = table_offset<PQL_BLOCK_BITS * b + 40, 6, 8>(k.w, col16);
        const float4 t43 = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(tab + kTBF) + boff);
        const float rq[4] = {rb[b] * t43.x, rb[b] * t43.y, rb[b] * t43.z, rb[b] * t43.w};
        H4 kq[4];
        kq[0].d = quarter_entry<PQL_BLOCK_BITS * b + 0, PQ_KEY_PAIRS != 0>(tab, k.w, col4);
        kq[1].d = quarter_entry<PQL_BLOCK_BITS * b + 10, PQ_KEY_PAIRS != 0>(tab, k.w, col4);
        kq[2].d = quarter_entry<PQL_BLOCK_BITS * b + 20, PQ_KEY_PAIRS != 0>(tab, k.w, col4);
        kq[3].d = quarter_entry<PQL_BLOCK_BITS * b + 30, PQ_KEY_PAIRS != 0>(tab, k.w, col4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            constexpr int set = b >> 2;         /* quarters 0..15 | 16..31 */
            const int abid = (4 * b + j) & 15;  /* compile-time after unrolling */
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                f4 d;
                switch (abid) { /* the broadcast selector is an immediate of the instruction */
#define PQ_SCORE_CASE(N)                                                                                     \
    case N:                                                                                                  \
        d = __builtin_amdgcn_mfma_f32_4x4x4f16(qo.a[g][set].v, kq[j].v, zero, 4, N, 0);                         \
        break;
                    PQ_SCORE_CASE(0) PQ_SCORE_CASE(1) PQ_SCORE_CASE(2) PQ_SCORE_CASE(3)
                    PQ_SCORE_CASE(4) PQ_SCORE_CASE(5) PQ_SCORE_CASE(6) PQ_SCORE_CASE(7)
                    PQ_SCORE_CASE(8) PQ_SCORE_CASE(9) PQ_SCORE_CASE(10) PQ_SCORE_CASE(11)
                    PQ_SCORE_CASE(12) PQ_SCORE_CASE(13) PQ_SCORE_CASE(14)
                    default: PQ_SCORE_CASE(15)
#undef PQ_SCORE_CASE
                }
#pragma unroll
                for (int h = 0; h < 4; ++h) s[g][h] = __builtin_fmaf(d[h], rq[j], s[g][h]);
            }
        }
    };
    block(std::integral_constant<int, 0>{}); block(std::integral_constant<int, 1>{});
    block(std::integral_constant<int, 2>{}); block(std::integral_constant<int, 3>{});
    block(std::integral_constant<int, 4>{}); block(std::integral_constant<int, 5>{});
    block(std::integral_constant<int, 6>{}); block(std::integral_constant<int, 7>{});
}

/* A operands of the weighted value sum of pass i: the rebuilt values of tokens 16 i + 4 g + e, e = 0..3, for
 * this lane's half-block, one operand per pair of coordinates c.  Per token: the radius times the block-table
 * entry of this half (one packed product: the two quarter radii), times the two quarter entries T21[Q]
 * (four packed products).  MASKED zeroes the radii of slots beyond the sequence's context so that stale
 * cache bytes there cannot reach the sum. */
template <int i, bool MASKED, bool DEEP>
__device__ __forceinline__ void value_operand(const uint32_t *tab, const char *tbh /* block table of the values */,
                                              const VTileRaw &v, H8 (&va)[4], int n_valid, int g, const DeepRadii &dr,
                                              int lane)
{
    uint32_t rpair[2]; /* radii of tokens (0, 1) and (2, 3) of the pass */
    if (DEEP) {
        const uint2 rr = *reinterpret_cast<const uint2 *>(dr.vrad + (lane >> 1) * 16 + 4 * i);
        rpair[0] = rr.x; rpair[1] = rr.y;
    } else {
        const uint4 rq = (i < 2) ? v.rad0 : v.rad1;
        rpair[0] = sel4(rq, 2 * (i & 1));
        rpair[1] = sel4(rq, 2 * (i & 1) + 1);
    }
    h2 ve[4][4]; /* [token e][pair c] */
    const uint32_t col4 = (uint32_t)(lane & 31) * 4u;
    auto token = [&](auto ec) {
        constexpr int e = decltype(ec)::value, s = 4 * i + e;
        const h2 rad = as_h2(rpair[e >> 1]);
        h2 r = (e & 1) ? bcast_hi(rad) : bcast_lo(rad);
        if (MASKED) {
            if (16 * i + 4 * g + e >= n_valid) r = h2{(_Float16)0.f, (_Float16)0.f};
        }
        const uint32_t boff = table_offset<6 * s, 6, 7>(v.b, col4);
        const h2 t43 = as_h2(*reinterpret_cast<const uint32_t *>(tbh + boff));
        const uint2 ta = quarter_entry<PQL_SLOT_BITS * s, PQ_VALUE_PAIRS != 0>(tab, v.q, col4);
        const uint2 tb = quarter_entry<PQL_SLOT_BITS * s + 10, PQ_VALUE_PAIRS != 0>(tab, v.q, col4);
        const h2 rq = r * t43; /* radii of the half-block's two quarters */
        const h2 ra = bcast_lo(rq), rbq = bcast_hi(rq);
        ve[e][0] = ra * as_h2(ta.x);
        ve[e][1] = ra * as_h2(ta.y);
        ve[e][2] = rbq * as_h2(tb.x);
        ve[e][3] = rbq * as_h2(tb.y);
    };
    token(std::integral_constant<int, 0>{}); token(std::integral_constant<int, 1>{});
    token(std::integral_constant<int, 2>{}); token(std::integral_constant<int, 3>{});
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) va[c].p[e] = ve[e][c];
}

__device__ __forceinline__ float wave_max_f(float x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d));
    return x;
}

/* G query heads per kv head, M query tokens per sequence (a.M), NG column groups with
 * M * G <= 4 * NG.  Query token m of a sequence is its (M-1-m)-th newest token and sees
 * the cache up to and including its own key: ctx - (M-1-m) tokens.
 *
 * Per 64-token tile: scores with one token per lane (key_scores), probabilities
 * p = 2^(s - m + kProbShift) against an exponent reference m per pair that only moves when a score
 * exceeds it by more than kRefSlack (wave-uniform test, rare after the first tile of a piece), the
 * probabilities handed through LDS to the layout of the value contraction (lane (g, column) needs
 * four consecutive tokens of one pair), then four passes of 16 tokens of weighted values on
 * v_mfma_f32_16x16x32_f16.  The (cos, sin)-like pairs of a table entry are two coordinates of one
 * token, while a matrix-core operand wants several tokens of one coordinate per lane; instead of
 * transposing, the contraction index is widened to (token, parity): operand rows are coordinate
 * pairs, and the probability operand has one column per (pair, parity) with zeros in the slots of
 * the other parity.  The result accumulates o' for the even coordinates in the parity-0 columns and
 * for the odd ones in parity 1. */
template <int NG, bool DEEP>
__global__ __launch_bounds__(waves_per_block(NG) * 64, 1) void pq_attn_partial_kernel(AttnArgs a)
{
    constexpr int kWavesPerBlock = waves_per_block(NG), kThreads = kWavesPerBlock * 64;
    const int G = a.Hq / a.Hkv; /* query heads per kv head: only the set-up and the epilogue of a piece depend on it */
    __shared__ __attribute__((aligned(16))) uint32_t tab[kLdsTabDwords];
    /* probabilities of a tile: sP[wave][group][column = pair slot + 4 parity][token] as dwords; a parity-0 column
       keeps its binary16 value in the low half, a parity-1 column in the high half, and the other halves stay
       zero from the start of the kernel (nothing ever writes them) */
    __shared__ __attribute__((aligned(16))) uint32_t sP[kWavesPerBlock][NG][8][64];
    __shared__ __attribute__((aligned(16))) uint16_t sVrad[DEEP ? kWavesPerBlock : 1][DEEP ? 512 : 8];
    /* per-sequence data of batches of up to 64 sequences is staged in LDS with the tables, so that
       nothing between the barrier and the first tile request waits for global memory; its loads
       are requested first (last wavefront of the workgroup) */
    /* tiles done so far by every wavefront, [wavefront & 3][wavefront >> 2]: the wavefronts of a workgroup go to the
       four SIMDs in turn, so a row holds the wavefronts that share a SIMD (see the issue priority in the tile loop) */
    __shared__ __attribute__((aligned(16))) int sDone[4][4];
    __shared__ int sPre[65];
    __shared__ int sCtx[64];
    __shared__ int64_t sTile0[64];
    const bool staged = a.B <= 64;
    const int total = a.plan[0], share = a.plan[1];
    int st_pre = 0, st_last = 0, st_len = 0;
    int64_t st_start = 0;
    constexpr int kStager = kThreads - 64; /* first thread of the last wavefront */
    if (staged && threadIdx.x >= kStager) {
        const int bb = (int)threadIdx.x - kStager;
        st_pre = a.plan[kPlanHeader + min(bb, a.B)];
        st_last = a.plan[kPlanHeader + a.B];
        st_len = a.ctx_len[min(bb, a.B - 1)];
        st_start = a.seq_start[min(bb, a.B - 1)];
    }
    {   /* tables: the image in global memory is compact (PQ_TAB_*); the small ones are spread over a column per lane.
           All of a thread's entries are requested before the first one is stored: one trip to memory, not one per
           entry. */
        const uint32_t *src = a.consts->attn_tab;
        constexpr int kR2 = (2048 + kThreads - 1) / kThreads, kR4 = (4096 + kThreads - 1) / kThreads;
        uint32_t tq[kR2], tqa[kR2], tqb[kR2], tbh[kR2], tbf[kR4], tup = 0;
#pragma unroll
        for (int i = 0; i < kR2; ++i) {
            const int t = min((int)threadIdx.x + i * kThreads, 2047); /* entry t >> 5, column t & 31 */
            tq[i] = src[PQ_TAB_TQ + t];
            tqa[i] = src[PQ_TAB_TQA + (t >> 5)];
            tqb[i] = src[PQ_TAB_TQB + (t >> 5)];
            tbh[i] = src[PQ_TAB_TBH + 2 * (t >> 5) + (t & 1)];
        }
#pragma unroll
        for (int i = 0; i < kR4; ++i) {
            const int t = min((int)threadIdx.x + i * kThreads, 4095); /* entry t >> 6, column (t >> 2) & 15, float t & 3 */
            tbf[i] = src[PQ_TAB_TBF + 4 * (t >> 6) + (t & 3)];
        }
        if (threadIdx.x < 48) tup = src[PQ_TAB_UP + threadIdx.x];
        uint4 *pz = reinterpret_cast<uint4 *>(&sP[0][0][0][0]);
        for (int t = threadIdx.x; t < kWavesPerBlock * NG * 8 * 64 / 4; t += kThreads) pz[t] = make_uint4(0, 0, 0, 0);
        if (threadIdx.x < 16) sDone[threadIdx.x >> 2][threadIdx.x & 3] = threadIdx.x < kWavesPerBlock ? 0 : 0x7FFFFFFF;
#pragma unroll
        for (int i = 0; i < kR2; ++i) {
            const int t = (int)threadIdx.x + i * kThreads;
            if (t < 2048) {
                tab[kTQ + t] = tq[i];
                tab[kTQA + t] = tqa[i];
                tab[kTQB + t] = tqb[i];
                tab[kTBH + t] = tbh[i];
            }
        }
#pragma unroll
        for (int i = 0; i < kR4; ++i) {
            const int t = (int)threadIdx.x + i * kThreads;
            if (t < 4096) tab[kTBF + t] = tbf[i];
        }
        if (threadIdx.x < 48) tab[kTUp + threadIdx.x] = tup;
    }
    if (staged && threadIdx.x >= kStager) {
        const int bb = (int)threadIdx.x - kStager;
        sPre[bb] = st_pre;
        if (bb == 63) sPre[64] = st_last;
        sCtx[bb] = bb < a.B ? effective_ctx_of(st_len, st_start, a.max_ctx, a.pool_tiles) : 0;
        sTile0[bb] = st_start >> 6;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    /* the wavefront index is the same in all lanes: telling the compiler so keeps everything
       derived from it (work range, pointers, loop bounds) in scalar registers */
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = (int)blockIdx.x * kWavesPerBlock + wave;
    if (share <= 0 || (int64_t)w * share >= total) return;
    int gpos = w * share;
    const int gend = min(gpos + share, total);
    /* wave-uniform reads of the per-sequence data (LDS values come back in vector registers:
       readfirstlane returns them to scalar ones) */
    auto prefix_at = [&](int i) -> int {
        return staged ? __builtin_amdgcn_readfirstlane(sPre[i]) : a.plan[kPlanHeader + i];
    };
    auto ctx_of = [&](int bb) -> int {
        return staged ? __builtin_amdgcn_readfirstlane(sCtx[bb])
                      : effective_ctx(a.seq_start, a.ctx_len, bb, a.max_ctx, a.pool_tiles);
    };
    auto tile0_of = [&](int bb) -> int64_t {
        if (!staged) return a.seq_start[bb] >> 6;
        const int64_t v = sTile0[bb];
        return (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
                         (uint32_t)__builtin_amdgcn_readfirstlane((int)v));
    };
    /* sequence of the first tile: the last b whose streams start at or before gpos (a ballot
       over the prefix table, 64 entries per round; empty sequences share their successor's entry) */
    int b;
    {
        int cnt = 0;
        if (staged) {
            cnt = __popcll(__ballot(lane <= a.B && (int64_t)sPre[lane] * a.Hkv <= gpos));
        } else {
            for (int base = 0; base <= a.B; base += 64) {
                const int i = base + lane;
                const bool at_or_before = i <= a.B && (int64_t)a.plan[kPlanHeader + min(i, a.B)] * a.Hkv <= gpos;
                cnt += __popcll(__ballot(at_or_before));
            }
        }
        b = min(max(cnt - 1, 0), a.B - 1);
    }
    int before = prefix_at(b);
    int seq_tiles = prefix_at(b + 1) - before;
    if (seq_tiles <= 0) return;
    int hk, tile_lo;
    {
        const int r = gpos - before * a.Hkv; /* below Hkv * seq_tiles */
        hk = min(r / seq_tiles, a.Hkv - 1);
        tile_lo = r - hk * seq_tiles;
    }
    const int g = lane >> 4, n = lane & 15;
    constexpr int kRadiiHalves = DEEP ? PQ_DEEP_RADII_HALVES : PQL_RADII;
    const DeepRadii dr{sVrad[DEEP ? wave : 0], a.up_b5, a.up_b6, a.up_b7};
    const char *tbh = reinterpret_cast<const char *>(tab + kTBH);
    /* where this lane (token) leaves its probabilities and where it (column) picks its operand up */
    uint32_t *p_mine = &sP[wave][0][0][lane];
    const uint32_t *p_col = &sP[wave][0][n & 7][4 * g];
    /* rotated queries and partial results: the launch code keeps all three below 4 GB */
    const __amdgpu_buffer_rsrc_t q_rsrc = stream_descriptor(a.qrot, (uint32_t)a.B * a.M * a.Hq * (PQ_D * 2u));
    const __amdgpu_buffer_rsrc_t o_rsrc = stream_descriptor(a.ws_o, (uint32_t)a.n_pieces * (a.M * G) * (PQ_D * 4u));
    const __amdgpu_buffer_rsrc_t ml_rsrc = stream_descriptor(a.ws_ml, (uint32_t)a.n_pieces * (a.M * G) * 8u);

    const int gpos0 = gpos;
    int *my_done = &sDone[wave & 3][wave >> 2];
    const int4 *simd_done = reinterpret_cast<const int4 *>(&sDone[wave & 3][0]);
    for (;;) { /* one piece per round: tiles [tile_lo, tile_hi) of stream (b, hk) */
        const int ctx = ctx_of(b);
        const int n_tiles = (ctx + 63) >> 6; /* == seq_tiles */
        const int tile_hi = min(n_tiles, tile_lo + (gend - gpos)); /* n_tiles bounds every read inside the pool */
        const int piece_tiles = tile_hi - tile_lo;
        if (piece_tiles <= 0) return; /* cannot happen with a consistent plan */
        const int64_t piece = (int64_t)w + (int64_t)b * a.Hkv + hk;

        const int64_t seq_tile0 = tile0_of(b);
        const int64_t stream_tile0 = (int64_t)hk * a.pool_tiles + seq_tile0;
        /* descriptors of this sequence's tiles in the four planes (the context is at most 2^31 tokens: 32-bit sizes) */
        const uint32_t code_bytes = (uint32_t)n_tiles * PQL_CODE_BYTES, radii_bytes = (uint32_t)n_tiles * (kRadiiHalves * 2u);
        const __amdgpu_buffer_rsrc_t kc = stream_descriptor(a.k_codes + stream_tile0 * PQL_CODE_BYTES, code_bytes);
        const __amdgpu_buffer_rsrc_t vc = stream_descriptor(a.v_codes + stream_tile0 * PQL_CODE_BYTES, code_bytes);
        const __amdgpu_buffer_rsrc_t kr = stream_descriptor(a.k_radii + stream_tile0 * kRadiiHalves, radii_bytes);
        const __amdgpu_buffer_rsrc_t vr = stream_descriptor(a.v_radii + stream_tile0 * kRadiiHalves, radii_bytes);

        /* ---- q' operands (see QueryOperand); pair p = (query token p / G, head p % G) ---- */
        QueryOperand<NG> qo;
        /* lane-dependent addresses of the piece's prologue and epilogue are formed from a copy of the lane
           number that the compiler cannot trace: hoisted out of the piece loop they would be spilled */
        int lane_q = lane;
        asm volatile("" : "+v"(lane_q));
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            const int slot = lane_q & 3, qi = lane_q >> 2;
            const int pair = 4 * k + slot;
            const bool real = pair < a.M * G;
            const int m = real ? pair / G : 0, head = real ? pair % G : 0;
            /* 32-bit offsets into the rotated queries: lane part in bytes, (sequence, kv head) part scalar */
            const uint32_t lane_off = (uint32_t)((m * a.Hq + head) * PQ_D + 4 * qi) * 2u;
            const uint32_t row_off = (uint32_t)((b * a.M * a.Hq + hk * G) * PQ_D) * 2u;
#pragma unroll
            for (int set = 0; set < 2; ++set) {
                const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(q_rsrc, lane_off + (uint32_t)(64 * set) * 2u, row_off, 0);
                qo.a[k][set].w[0] = real ? v.x : 0u;
                qo.a[k][set].w[1] = real ? v.y : 0u;
            }
        }
        f4 acc_o[NG][4];
        /* exponent reference of a pair: the same in all lanes; l: this lane's share of the sum of its token's weights */
        float m_ref[NG][4], l_run[NG][4];
#pragma unroll
        for (int k = 0; k < NG; ++k) {
#pragma unroll
            for (int c = 0; c < 4; ++c) acc_o[k][c] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int h = 0; h < 4; ++h) { m_ref[k][h] = 0.f; l_run[k][h] = 0.f; }
        }
        bool have_ref = false; /* m_ref is a place holder until the first tile of the piece has set it */

        /* One tile.  MASKED: the tile holds tokens beyond the context, or beyond what one of the query
         * tokens may see (lim[k][h]: tokens of this tile that pair 4 k + h sees; nv: tokens inside the context). */
        auto do_tile = [&](auto masked_c, const KTileRaw &kraw, const VTileRaw &vraw, const int (&lim)[NG][4], int nv) {
            constexpr bool MASKED = decltype(masked_c)::value;
            float s[NG][4];
#pragma unroll
            for (int k = 0; k < NG; ++k)
#pragma unroll
                for (int h = 0; h < 4; ++h) s[k][h] = kProbShift - m_ref[k][h];
            key_scores<NG, DEEP>(tab, kraw, qo, s, dr, lane); /* s = score - m_ref + kProbShift */
            if (MASKED) {
#pragma unroll
                for (int k = 0; k < NG; ++k)
#pragma unroll
                    for (int h = 0; h < 4; ++h)
                        if (lane >= lim[k][h]) s[k][h] = -INFINITY;
            }
            float top = s[0][0];
#pragma unroll
            for (int k = 0; k < NG; ++k)
#pragma unroll
                for (int h = 0; h < 4; ++h) top = fmaxf(top, s[k][h]);
            if (!have_ref || __ballot(top > kProbShift + kRefSlack) != 0ull) { /* wave-uniform */
#pragma unroll
                for (int k = 0; k < NG; ++k) {
                    float alpha_lane = 1.f; /* factor of this lane's output column (pair n & 3 of the group) */
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const float smax = __builtin_amdgcn_readfirstlane(wave_max_f(s[k][h]));
                        /* move the reference so that the largest weight of the tile is 2^kProbShift; a pair that has
                           seen no token yet (smax == -inf) keeps its place holder */
                        float delta = smax == -INFINITY ? 0.f : smax - kProbShift;
                        if (have_ref) delta = fmaxf(delta, 0.f);
                        const float alpha = have_ref ? __builtin_amdgcn_exp2f(-delta) : 1.f; /* nothing accumulated yet */
                        m_ref[k][h] += delta;
                        s[k][h] -= delta;
                        l_run[k][h] *= alpha;
                        if ((n & 3) == h) alpha_lane = alpha;
                    }
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc_o[k][c] *= alpha_lane;
                }
                have_ref = true;
            }
            wave_lds_fence(); /* the passes of the previous tile have read their operands */
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                _Float16 ph[4];
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const float p = __builtin_amdgcn_exp2f(s[k][h]); /* exp2(-inf) = 0 for masked tokens */
                    l_run[k][h] += p;
                    ph[h] = (_Float16)p;
                }
                _Float16 *dst = reinterpret_cast<_Float16 *>(p_mine + k * (8 * 64));
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    dst[2 * (h * 64)] = ph[h];                /* column (h, parity 0): low half */
                    dst[2 * ((4 + h) * 64) + 1] = ph[h];      /* column (h, parity 1): high half */
                }
            }
            if (DEEP) stage_deep_value_radii(tab, dr, vraw.top, lane);
            wave_lds_fence();
            auto pass = [&](auto ic) {
                constexpr int i = decltype(ic)::value;
                H8 va[4];
                value_operand<i, MASKED, DEEP>(tab, tbh, vraw, va, nv, g, dr, lane);
#pragma unroll
                for (int k = 0; k < NG; ++k) {
                    H8 pb;
                    pb.q = *reinterpret_cast<const uint4 *>(p_col + k * (8 * 64) + 16 * i);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        acc_o[k][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va[c].v, pb.v, acc_o[k][c], 0, 0, 0);
                }
            };
            pass(std::integral_constant<int, 0>{}); pass(std::integral_constant<int, 1>{});
            pass(std::integral_constant<int, 2>{}); pass(std::integral_constant<int, 3>{});
        };

        /* Tiles tile_lo .. tile_hi-1.  A tile is full when every query token sees all of its 64
         * tokens; the tiles after that (the sequence's last one, or its last two when the M newest
         * tokens straddle a tile boundary) are masked per pair.
         * The raw tile registers are single buffered: the next tiles are requested once the
         * last pass has consumed the current ones; the other wavefronts resident on the SIMD cover the latency. */
        const int n_full = min(tile_hi, max(ctx - (a.M - 1), 0) >> 6);
        KTileRaw kraw;
        VTileRaw vraw;
        load_k_tile<DEEP>(kraw, kc, kr, tile_lo, lane);
        load_v_tile<DEEP>(vraw, vc, vr, tile_lo, lane);
        int tile = tile_lo;
        {
            int lim[NG][4];
#pragma unroll
            for (int k = 0; k < NG; ++k)
#pragma unroll
                for (int h = 0; h < 4; ++h) lim[k][h] = 64;
            for (; tile < n_full; ++tile) {
                /* Issue priority by rank among the wavefronts of the SIMD: the hardware prefers the oldest, which
                   would run ahead and leave the youngest to finish alone at a fraction of the SIMD's issue rate.
                   Every wavefront publishes the tiles it has done; the more of its neighbours are ahead of it, the
                   higher its priority (a slot without a wavefront counts as infinitely far ahead). */
                {
                    const int done = gpos - gpos0 + (tile - tile_lo);
                    if (lane == 0) *my_done = done;
                    const int4 d4 = *simd_done;
                    const int ahead = (d4.x > done) + (d4.y > done) + (d4.z > done) + (d4.w > done);
                    set_wave_priority(min(__builtin_amdgcn_readfirstlane(ahead), 3));
                }
                do_tile(std::false_type{}, kraw, vraw, lim, 64);
                if (tile + 1 < tile_hi) {
                    load_k_tile<DEEP>(kraw, kc, kr, tile + 1, lane);
                    load_v_tile<DEEP>(vraw, vc, vr, tile + 1, lane);
                }
            }
        }
        for (; tile < tile_hi; ++tile) { /* the masked tiles at the end of the sequence */
            const int nv = min(ctx - tile * 64, 64);
            int lim[NG][4]; /* tokens of this tile that pair 4 k + h may see */
#pragma unroll
            for (int k = 0; k < NG; ++k)
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const int pair = 4 * k + h;
                    const int m = pair < a.M * G ? pair / G : 0;
                    lim[k][h] = ctx - (a.M - 1 - m) - tile * 64;
                }
            do_tile(std::true_type{}, kraw, vraw, lim, nv);
            if (tile + 1 < tile_hi) {
                load_k_tile<DEEP>(kraw, kc, kr, tile + 1, lane);
                load_v_tile<DEEP>(vraw, vc, vr, tile + 1, lane);
            }
        }

        /* ---- partial results: l summed over the tokens (lanes); o' scattered to coordinate order ---- */
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            float l_pair[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                float l = l_run[k][h];
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) l += __shfl_xor(l, d); /* the same order in every lane */
                l_pair[h] = l;
            }
            const int ne = lane_e & 15, ge = lane_e >> 4;
            const int pair = 4 * k + (ne & 3);
            if (ne < 8 && pair < a.M * G) {
                const int par = (ne >> 2) & 1;
                /* stores through descriptors as well: scalar piece offset, 32-bit lane offset */
                const uint32_t piece_o = (uint32_t)piece * (uint32_t)(a.M * G) * (PQ_D * 4u);
                const uint32_t lane_o = (uint32_t)(pair * PQ_D + 2 * 16 * ge + par) * 4u;
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc_o[k][c][e]), o_rsrc,
                                                              lane_o + 8u * (4 * e + c), piece_o, 0);
                if (ge == 0 && par == 0) {
                    const int h = ne & 3;
                    const float mm = h == 0 ? m_ref[k][0] : (h == 1 ? m_ref[k][1] : (h == 2 ? m_ref[k][2] : m_ref[k][3]));
                    const float ll = h == 0 ? l_pair[0] : (h == 1 ? l_pair[1] : (h == 2 ? l_pair[2] : l_pair[3]));
                    const uint32_t piece_ml = (uint32_t)piece * (uint32_t)(a.M * G) * 8u;
                    /* a pair that saw no token reports (-inf, 0), which the combine step drops */
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(ll > 0.f ? mm : -INFINITY), ml_rsrc, pair * 8u, piece_ml, 0);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(ll), ml_rsrc, pair * 8u + 4u, piece_ml, 0);
                }
            }
        }

        /* next piece: the first tiles of the next non-empty stream, as far as this wavefront's range goes */
        gpos += piece_tiles;
        if (gpos >= gend) return;
        tile_lo = 0;
        if (++hk == a.Hkv) {
            hk = 0;
            do {
                if (++b >= a.B) return; /* cannot happen: gpos < total */
                before = prefix_at(b);
                seq_tiles = prefix_at(b + 1) - before;
            } while (seq_tiles <= 0);
        }
    }
}

struct RotateArgs {
    const uint16_t *q; /* bf16 [rows][128] */
    uint16_t *qrot;    /* binary16 [rows][128] */
    const float *S;    /* S[i*128 + j] */
    float scale;       /* softmax_scale * log2(e) */
    const PqDeviceConsts *consts;
    PqHadamard had;    /* on: q' = q S by a fast Walsh-Hadamard transform, S is not read */
};

/* Four query rows per workgroup: the workgroup's slice of S (64 KB, what bounds this launch) is
 * fetched once for the four.  Thread (kq, j) accumulates the quarter kq of the sum over i for
 * column j of each row; thread (r, j) then adds the four quarters of row r in a fixed order
 * (the same order as vector_times_slice). */
constexpr int kRotateRows = 4;

__device__ __forceinline__ void rotate_query_rows(const RotateArgs &a, int row0, int n_rows)
{
    __shared__ float sq[kRotateRows][PQ_D];
    __shared__ float spart[kRotateRows][4][PQ_D];
    const int tid = threadIdx.x, r = tid >> 7, j = tid & 127;
    if (a.had.on) { /* S = D H / sqrt(128): wavefront w transforms row row0 + w, two elements per lane */
        const int w = tid >> 6, lane = tid & 63, hrow = row0 + w;
        if (w < kRotateRows && hrow < n_rows) {
            const uint16_t *qr = a.q + (int64_t)hrow * PQ_D;
            float lo = __uint_as_float((uint32_t)qr[lane] << 16) * pq_hadamard_sign(a.had, lane);
            float hi = __uint_as_float((uint32_t)qr[lane + 64] << 16) * pq_hadamard_sign(a.had, lane + 64);
            pq_fwht128(lo, hi, lane);
            const float c = a.scale * PQ_INV_SQRT_D;
            a.qrot[(int64_t)hrow * PQ_D + lane] = __builtin_bit_cast(uint16_t, (_Float16)(lo * c));
            a.qrot[(int64_t)hrow * PQ_D + lane + 64] = __builtin_bit_cast(uint16_t, (_Float16)(hi * c));
        }
        return;
    }
    MatrixSlice ms;
    matrix_slice_load(ms, a.S, tid);
    const int row = row0 + r;
    sq[r][j] = row < n_rows ? __uint_as_float((uint32_t)a.q[(int64_t)row * PQ_D + j] << 16) : 0.f;
    __syncthreads();
    {
        const int kq = r; /* the same thread index split serves as (quarter, column) here */
        float acc[kRotateRows];
#pragma unroll
        for (int rr = 0; rr < kRotateRows; ++rr) acc[rr] = 0.f;
#pragma unroll
        for (int k = 0; k < 32; ++k)
#pragma unroll
            for (int rr = 0; rr < kRotateRows; ++rr) acc[rr] = fmaf(sq[rr][32 * kq + k], ms.m[k], acc[rr]); /* q'_j = sum_i q_i S[i][j] */
#pragma unroll
        for (int rr = 0; rr < kRotateRows; ++rr) spart[rr][kq][j] = acc[rr];
    }
    __syncthreads();
    if (row < n_rows) {
        const float acc = ((spart[r][0][j] + spart[r][1][j]) + spart[r][2][j]) + spart[r][3][j];
        const float v = acc * a.scale;
        a.qrot[(int64_t)row * PQ_D + j] = __builtin_bit_cast(uint16_t, (_Float16)v);
    }
}

struct PlanArgs {
    const int64_t *seq_start;
    const int32_t *ctx_len;
    int B, Hkv;
    int64_t max_ctx, pool_tiles;
    int slots;     /* wavefronts of the partial kernel's launch */
    int32_t *plan; /* [kPlanHeader + (B + 1) + 2 * B * Hkv] */
};

/* Builds the work plan (one workgroup of 512 threads): running sum of the sequences' tile
 * counts, 512 sequences per round (a shuffle scan inside each wavefront, then the
 * wavefronts' totals), the total and the share of a wavefront, and from those the first
 * wavefront and the piece count of every stream. */
__device__ __forceinline__ void build_plan(const PlanArgs &a)
{
    __shared__ int wave_sum[8];
    __shared__ int s_share;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int carry = 0;
    for (int base = 0; base < a.B; base += 512) {
        const int b = base + tid;
        int v = b < a.B ? (effective_ctx(a.seq_start, a.ctx_len, b, a.max_ctx, a.pool_tiles) + 63) >> 6 : 0;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(v, d);
            if (lane >= d) v += up;
        }
        if (lane == 63) wave_sum[wv] = v;
        __syncthreads();
        int offset = carry, round_total = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int ws = wave_sum[k];
            if (k < wv) offset += ws;
            round_total += ws;
        }
        if (b < a.B) a.plan[kPlanHeader + b + 1] = offset + v;
        carry += round_total;
        __syncthreads();
    }
    if (tid == 0) {
        const uint32_t total = (uint32_t)carry * (uint32_t)a.Hkv;
        uint32_t share = (total + (uint32_t)a.slots - 1u) / (uint32_t)a.slots;
        if (share < (uint32_t)kMinShareTiles) share = kMinShareTiles;
        a.plan[0] = (int)total;
        a.plan[1] = (int)share;
        a.plan[kPlanHeader] = 0;
        s_share = (int)share;
    }
    __syncthreads(); /* also orders this workgroup's plan[] stores before the loads below */
    const uint32_t share = (uint32_t)s_share;
    int32_t *streams = a.plan + kPlanHeader + a.B + 1;
    for (int s = tid; s < a.B * a.Hkv; s += 512) {
        const int b = s / a.Hkv, hk = s - b * a.Hkv;
        const uint32_t before = (uint32_t)a.plan[kPlanHeader + b];
        const uint32_t seq_tiles = (uint32_t)a.plan[kPlanHeader + b + 1] - before;
        const uint32_t first_tile = before * (uint32_t)a.Hkv + (uint32_t)hk * seq_tiles; /* in the global tile sequence */
        const uint32_t w_first = first_tile / share;
        streams[2 * s] = (int)w_first;
        streams[2 * s + 1] = seq_tiles > 0 ? (int)((first_tile + seq_tiles - 1) / share - w_first) + 1 : 0;
    }
}

/* workgroups [0, row_blocks) rotate kRotateRows query rows each, the last workgroup builds the work plan */
__global__ __launch_bounds__(512) void pq_rotate_q_kernel(RotateArgs a, PlanArgs p, int rows, int row_blocks)
{
    if ((int)blockIdx.x < row_blocks) rotate_query_rows(a, kRotateRows * (int)blockIdx.x, rows);
    else build_plan(p);
}

/* First launch of a whole decode step: workgroups [0, n) append the new key vectors,
   [n, 2n) the new value vectors, the next row_blocks rotate kRotateRows query rows each and the
   last one builds the work plan; the jobs are independent of each other and all of them precede
   the attention proper. */
template <int XT>
__global__ __launch_bounds__(512) void pq_step_prologue_kernel(RotateArgs r, AppendArgs k, AppendArgs v, int n,
                                                               PlanArgs p, int rows, int row_blocks)
{
    const int blk = (int)blockIdx.x;
    if (blk < n) append_vector<XT>(k, PQ_KEY, blk);
    else if (blk < 2 * n) append_vector<XT>(v, PQ_VALUE, blk - n);
    else if (blk < 2 * n + row_blocks) rotate_query_rows(r, kRotateRows * (blk - 2 * n), rows);
    else build_plan(p);
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d));
    return x;
}

struct CombineArgs {
    const float *ws_ml, *ws_o; /* [piece][M * G pairs][2], [piece][M * G pairs][128] */
    int B, Hq, Hkv, M; /* rows are ordered [B][M][Hq] */
    const int32_t *plan;
    const float *St; /* St[j*128 + i] = S[i][j] */
    void *out;       /* bf16 or f32 [B][Hq][128] */
    int out_f32;
    const PqDeviceConsts *consts;
    /* unquantised window (hybrid attention only): partial results in the original domain */
    const float *win_ml, *win_o;
    const int32_t *win_len;
    int n_wchunks, win_cap;
    PqHadamard had; /* on: the un-rotation by S^T is a fast Walsh-Hadamard transform, St is not read */
};

/* HYBRID adds the partial results of the unquantised window.  They live in the original
 * domain, so they join after the un-rotation of the prefix sum:
 * out = (S^T-product of (sum_c w_c o'_c) + sum_w w_w o_w) / (sum of all w l). */
template <bool HYBRID>
__global__ __launch_bounds__(512) void pq_attn_combine_kernel(CombineArgs a)
{
    __shared__ float so[PQ_D];
    __shared__ float spart[4][PQ_D];
    __shared__ float sl[4][PQ_D];
    __shared__ float sw[4][PQ_D];
    const int tid = threadIdx.x, cq = tid >> 7, j = tid & 127;
    const int row = blockIdx.x;
    MatrixSlice ms; /* requested first: its latency overlaps the reads of the partial results */
    if (!a.had.on) matrix_slice_load(ms, a.St, tid);
    const int b = row / (a.M * a.Hq), mq = (row / a.Hq) % a.M, head = row % a.Hq;
    /* the pieces of this row's stream (sequence b, kv head hk): the wavefronts whose tile ranges
       meet the stream's, in order; their ids are consecutive.  A piece beyond what query token
       mq may see carries (m, l) = (-inf, 0) and drops out below. */
    const int G = a.Hq / a.Hkv, hk = head / G, pairs = a.M * G, pair = mq * G + head % G;
    const int s_index = b * a.Hkv + hk;
    const int32_t *stream = a.plan + kPlanHeader + a.B + 1 + 2 * s_index;
    const int w_first = stream[0], used = stream[1];
    const int64_t slot0 = ((int64_t)w_first + s_index) * pairs + pair;
    const int64_t ml_stride = 2 * (int64_t)pairs, o_stride = (int64_t)pairs * PQ_D;
    const float *ml = a.ws_ml + slot0 * 2;
    const float *op = a.ws_o + slot0 * PQ_D + j;
    int used_w = 0;
    const float *wml = nullptr, *wop = nullptr;
    if (HYBRID) {
        int w = a.win_len[b];
        w = w < 0 ? 0 : (w > a.win_cap ? a.win_cap : w);
        used_w = (w + 63) >> 6;
        wml = a.win_ml + (int64_t)row * a.n_wchunks * 2;
        wop = a.win_o + (int64_t)row * a.n_wchunks * PQ_D + j;
    }
    /* overall maximum first (every wavefront on its own: lane i reads the maximum of piece i, 64 + i, ...,
       so the reads are in flight together), then the weighted sums; thread group cq takes chunks cq, cq+4, ...
       and the four group sums are added in a fixed order: the result does not depend on scheduling */
    float m = -INFINITY;
    {
        const int lane = tid & 63;
        for (int c = lane; c < used; c += 64) m = fmaxf(m, ml[c * ml_stride]);
        if (HYBRID)
            for (int c = lane; c < used_w; c += 64) m = fmaxf(m, wml[2 * c]);
        m = wave_max(m);
    }
    float l = 0.f, o = 0.f, ow = 0.f;
    if (m != -INFINITY) {
#pragma unroll 4
        for (int c = cq; c < used; c += 4) {
            const float w = exp2f(ml[c * ml_stride] - m);
            l = fmaf(ml[c * ml_stride + 1], w, l);
            o = fmaf(op[c * o_stride], w, o);
        }
    }
    if (HYBRID) {
        for (int c = cq; c < used_w; c += 4) {
            const float w = exp2f(wml[2 * c] - m);
            l = fmaf(wml[2 * c + 1], w, l);
            ow = fmaf(wop[(int64_t)c * PQ_D], w, ow);
        }
        sw[cq][j] = ow;
    }
    spart[cq][j] = o;
    sl[cq][j] = l;
    __syncthreads();
    float lt = 0.f, owt = 0.f;
    if (tid < PQ_D) {
        const float ot = ((spart[0][j] + spart[1][j]) + spart[2][j]) + spart[3][j];
        lt = ((sl[0][j] + sl[1][j]) + sl[2][j]) + sl[3][j];
        if (HYBRID) {
            owt = ((sw[0][j] + sw[1][j]) + sw[2][j]) + sw[3][j];
            so[j] = ot;
        } else {
            so[j] = lt > 0.f ? ot / lt : 0.f; /* lt == 0: no visible token */
        }
    }
    __syncthreads();
    float acc; /* out_j = sum_k o'_k S[j][k] */
    if (a.had.on) { /* = D_j / sqrt(128) times the Walsh-Hadamard transform of o' */
        if (tid < 64) {
            float lo = so[tid], hi = so[tid + 64];
            pq_fwht128(lo, hi, tid);
            spart[0][tid] = lo * PQ_INV_SQRT_D * pq_hadamard_sign(a.had, tid);
            spart[0][tid + 64] = hi * PQ_INV_SQRT_D * pq_hadamard_sign(a.had, tid + 64);
        }
        __syncthreads();
        acc = spart[0][j];
    } else {
        acc = vector_times_slice(so, ms, spart, tid);
    }
    if (tid < PQ_D) {
        if (HYBRID) acc = lt > 0.f ? (acc + owt) / lt : 0.f;
        if (a.out_f32) {
            static_cast<float *>(a.out)[(int64_t)row * PQ_D + j] = acc;
        } else {
            uint32_t u = __float_as_uint(acc);
            static_cast<uint16_t *>(a.out)[(int64_t)row * PQ_D + j] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
        }
    }
}

/* ---- unquantised recent window (Section 5.3: generation-stage keys and values stay in
 * 16 bits): plain attention partials over bf16 rows, in the original domain.  One wavefront
 * per (sequence, kv head, chunk of 64 window tokens); lane t scores token t against the G
 * query heads of the group (q in LDS, read as broadcasts), the wavefront reduces maximum
 * and sum, then lane c accumulates coordinates 2c, 2c+1 of the weighted value sum with the
 * value rows read as whole 256-byte lines.  The window is short next to the quantised
 * prefix, so this kernel is kept simple (vector ALU only). */
struct WindowArgs {
    const uint16_t *q;      /* bf16 [B][Hq][128] */
    const uint16_t *win_k;  /* bf16 [B][Hkv][win_cap][128] */
    const uint16_t *win_v;
    const int32_t *win_len; /* [B] */
    int B, Hq, Hkv, win_cap, n_wchunks;
    float scale;            /* softmax_scale * log2(e) */
    float *win_ml;          /* [B][Hq][n_wchunks][2] */
    float *win_o;           /* [B][Hq][n_wchunks][128] */
};

__device__ __forceinline__ float wave_sum_fixed(float x)
{
    /* butterfly: every lane adds the same pairs in the same order, the result is reproducible */
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
    return x;
}

/* G = query heads handled by one wavefront: the group of a kv head (Hq/Hkv), or half of it when the group
   has four heads -- the kernel has little work per launch and runs faster spread over more wavefronts */
constexpr int kWindowWaves = 4; /* work items per workgroup: one per SIMD, as many workgroups as possible */

template <int G>
__device__ __forceinline__ void window_item(const WindowArgs &a, int64_t item, int wave, int lane,
                                            float (&sq)[kWindowWaves][G][PQ_D], float (&sp)[kWindowWaves][G][64])
{
    const int n_hg = a.Hq / G; /* head groups of G heads; head0 = first query head of this wavefront */
    const int wc = (int)(item % a.n_wchunks);
    const int head0 = (int)((item / a.n_wchunks) % n_hg) * G;
    const int hk = head0 / (a.Hq / a.Hkv);
    const int b = (int)(item / ((int64_t)a.n_wchunks * n_hg));
    if (b >= a.B) return;
    int W = a.win_len[b];
    W = W < 0 ? 0 : (W > a.win_cap ? a.win_cap : W);
    const int t0 = 64 * wc;
    const int n_valid = min(W - t0, 64);
    if (n_valid <= 0) return; /* the combine kernel reads only the chunks below win_len */

    /* q of the group's heads, scaled, as fp32 in LDS */
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const uint32_t two = reinterpret_cast<const uint32_t *>(a.q + ((int64_t)b * a.Hq + head0 + h) * PQ_D)[lane];
        sq[wave][h][2 * lane] = __uint_as_float(two << 16) * a.scale;
        sq[wave][h][2 * lane + 1] = __uint_as_float(two & 0xFFFF0000u) * a.scale;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    /* scores: lane t takes window token t0 + t (lanes beyond the window re-read the last row) */
    const int64_t plane = ((int64_t)b * a.Hkv + hk) * a.win_cap;
    const int tl = lane < n_valid ? lane : n_valid - 1;
    const uint4 *krow = reinterpret_cast<const uint4 *>(a.win_k + (plane + t0 + tl) * PQ_D);
    float s[G];
#pragma unroll
    for (int h = 0; h < G; ++h) s[h] = 0.f;
    uint4 krow_v[16]; /* the whole 256-byte row is requested at once: one memory round trip */
#pragma unroll
    for (int c = 0; c < 16; ++c) krow_v[c] = krow[c];
#pragma unroll
    for (int c = 0; c < 16; ++c) { /* 8 coordinates per step */
        const uint4 kv = krow_v[c];
        const uint32_t w[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float4 qa = *reinterpret_cast<const float4 *>(&sq[wave][h][8 * c]);
            const float4 qb = *reinterpret_cast<const float4 *>(&sq[wave][h][8 * c + 4]);
            float acc = s[h];
            acc = fmaf(__uint_as_float(w[0] << 16), qa.x, acc);
            acc = fmaf(__uint_as_float(w[0] & 0xFFFF0000u), qa.y, acc);
            acc = fmaf(__uint_as_float(w[1] << 16), qa.z, acc);
            acc = fmaf(__uint_as_float(w[1] & 0xFFFF0000u), qa.w, acc);
            acc = fmaf(__uint_as_float(w[2] << 16), qb.x, acc);
            acc = fmaf(__uint_as_float(w[2] & 0xFFFF0000u), qb.y, acc);
            acc = fmaf(__uint_as_float(w[3] << 16), qb.z, acc);
            acc = fmaf(__uint_as_float(w[3] & 0xFFFF0000u), qb.w, acc);
            s[h] = acc;
        }
    }
    float m[G], l[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float sv = lane < n_valid ? s[h] : -INFINITY;
        m[h] = wave_max(sv);
        /* the same factor 2^kProbShift as the partial results of the quantised prefix carry */
        const float p = lane < n_valid ? __builtin_amdgcn_exp2f(sv - m[h] + kProbShift) : 0.f;
        l[h] = wave_sum_fixed(p);
        sp[wave][h][lane] = p;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    /* weighted values: lane c owns coordinates 2c, 2c+1; tokens in order */
    const uint32_t *vbase = reinterpret_cast<const uint32_t *>(a.win_v + (plane + t0) * PQ_D) + lane;
    float o0[G], o1[G];
#pragma unroll
    for (int h = 0; h < G; ++h) { o0[h] = 0.f; o1[h] = 0.f; }
    for (int tb = 0; tb < n_valid; tb += 8) { /* eight value rows in flight; rows beyond the window re-read the last one with weight 0 */
        uint32_t two[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) two[k] = vbase[(int64_t)min(tb + k, n_valid - 1) * (PQ_D / 2)];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float v0 = __uint_as_float(two[k] << 16), v1 = __uint_as_float(two[k] & 0xFFFF0000u);
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float p = tb + k < n_valid ? sp[wave][h][tb + k] : 0.f;
                o0[h] = fmaf(p, v0, o0[h]);
                o1[h] = fmaf(p, v1, o1[h]);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const int64_t slot = ((int64_t)b * a.Hq + head0 + h) * a.n_wchunks + wc;
        reinterpret_cast<float2 *>(a.win_o + slot * PQ_D)[lane] = make_float2(o0[h], o1[h]);
        if (lane == 0) {
            a.win_ml[slot * 2] = m[h];
            a.win_ml[slot * 2 + 1] = l[h];
        }
    }
}

/* First launch of hybrid attention: workgroups [0, wblocks) take four window items each (the first four
   wavefronts; these are the longest jobs of the launch, so they start first), the next row_blocks rotate
   the queries, the last one builds the work plan.  The window partials need the original queries only,
   so they share this launch instead of taking one of their own before it. */
template <int G>
__global__ __launch_bounds__(512) void pq_rotate_window_kernel(RotateArgs r, PlanArgs p, int rows, int row_blocks, WindowArgs w,
                                                               int wblocks)
{
    const int blk = (int)blockIdx.x;
    if (blk < wblocks) {
        __shared__ float sq[kWindowWaves][G][PQ_D];
        __shared__ float sp[kWindowWaves][G][64];
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        if (wave < kWindowWaves) window_item<G>(w, (int64_t)blk * kWindowWaves + wave, wave, lane, sq, sp);
    } else if (blk < wblocks + row_blocks) {
        rotate_query_rows(r, kRotateRows * (blk - wblocks), rows);
    } else {
        build_plan(p);
    }
}

struct Plan {
    int slots;       /* wavefronts of the partial kernel's launch */
    unsigned blocks; /* its workgroups */
    size_t off_plan, off_ml, off_o, total;
    size_t pieces, o_bytes; /* piece ids run below `pieces`; bytes of their o' */
    /* window partials (hybrid attention; n_wchunks == 0 otherwise) */
    int n_wchunks;
    size_t off_wml, off_wo;
};

/* Workspace: rotated queries | work plan | (m, l) of every piece | o' of every piece | window partials. */
Plan make_plan(int B, int Hq, int Hkv, int64_t max_ctx, int64_t win_cap = 0, int M = 1)
{
    Plan p;
    int64_t max_tiles = (max_ctx + 63) / 64;
    if (max_tiles < 1) max_tiles = 1;
    const int G = Hq / Hkv > 0 ? Hq / Hkv : 1;
    const int pairs = M * G;
    /* One wavefront per resident slot: 256 CUs x 4 SIMDs x the wavefronts per SIMD the kernel variant's
       register budget allows.  Every wavefront gets an equal share of the tiles (see DevicePlan above), so one
       round of resident wavefronts does the whole job and all of them finish together; more, smaller
       work items measured slower on the 32k-context batch (143 us against 149-156 us for 3/2 or 2 times
       as many) and write more partial results.  Small problems: no more wavefronts than shares of
       kMinShareTiles tiles. */
    const int per_simd = pairs <= 4 ? 4 : (pairs <= 8 ? 3 : 2);
    int64_t slots = 256 * 4 * per_simd;
    const int64_t most = ((int64_t)B * Hkv * max_tiles + kMinShareTiles - 1) / kMinShareTiles;
    if (slots > most) slots = most;
    const int block_waves = 4 * per_simd; /* = waves_per_block of the variant: one workgroup fills a CU */
    p.blocks = (unsigned)((slots + block_waves - 1) / block_waves);
    p.slots = (int)(p.blocks * block_waves);
    const size_t pieces = (size_t)p.slots + (size_t)B * Hkv; /* ids run below slots + streams */
    p.pieces = pieces;
    p.o_bytes = pieces * pairs * PQ_D * sizeof(float);
    size_t rows = (size_t)B * M * Hq;
    p.off_plan = (rows * PQ_D * sizeof(uint16_t) + 255) & ~(size_t)255;
    p.off_ml = (p.off_plan + (kPlanHeader + (size_t)B + 1 + 2 * (size_t)B * Hkv) * sizeof(int32_t) + 255) & ~(size_t)255;
    p.off_o = (p.off_ml + pieces * pairs * 2 * sizeof(float) + 255) & ~(size_t)255;
    p.total = p.off_o + pieces * pairs * PQ_D * sizeof(float);
    p.n_wchunks = (int)((win_cap + 63) / 64);
    p.off_wml = (p.total + 255) & ~(size_t)255;
    p.off_wo = (p.off_wml + rows * p.n_wchunks * 2 * sizeof(float) + 255) & ~(size_t)255;
    if (p.n_wchunks > 0) p.total = p.off_wo + rows * p.n_wchunks * PQ_D * sizeof(float);
    return p;
}

} // namespace

extern "C" const char *pq_kernel_name_attn(void) { return "pq_attn_partial_kernel"; }

extern "C" size_t pq_attn_workspace_bytes(int B, int Hq, int Hkv, int64_t max_ctx)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || max_ctx < 0) return 0;
    return make_plan(B, Hq, Hkv, max_ctx).total;
}

extern "C" size_t pq_attn_mq_workspace_bytes(int B, int M, int Hq, int Hkv, int64_t max_ctx)
{
    if (B <= 0 || M <= 0 || Hq <= 0 || Hkv <= 0 || max_ctx < 0) return 0;
    return make_plan(B, Hq, Hkv, max_ctx, 0, M).total;
}

extern "C" size_t pq_attn_hybrid_workspace_bytes(int B, int Hq, int Hkv, int64_t max_ctx, int64_t win_cap)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || max_ctx < 0 || win_cap < 0) return 0;
    return make_plan(B, Hq, Hkv, max_ctx, win_cap).total;
}

namespace {

/* the new key / value vectors of a decode step, appended by the first launch (optional) */
struct StepAppend {
    const void *xk, *xv;
    pq_dtype xt;
    const int64_t *dst_token;
    int n_heads;
};

/* the unquantised recent window of hybrid attention (optional) */
struct StepWindow {
    const void *win_k, *win_v;
    const int32_t *win_len;
    int64_t win_cap;
};

template <bool DEEP>
void launch_partial_depth(int NG, dim3 grid, dim3 blk, hipStream_t s, const AttnArgs &aa)
{
    if (NG == 1) hipLaunchKernelGGL((pq_attn_partial_kernel<1, DEEP>), grid, blk, 0, s, aa);
    else if (NG == 2) hipLaunchKernelGGL((pq_attn_partial_kernel<2, DEEP>), grid, blk, 0, s, aa);
    else hipLaunchKernelGGL((pq_attn_partial_kernel<4, DEEP>), grid, blk, 0, s, aa);
}

void launch_partial(int NG, bool deep, dim3 grid, dim3 blk, hipStream_t s, const AttnArgs &aa)
{
    if (deep) launch_partial_depth<true>(NG, grid, blk, s, aa);
    else launch_partial_depth<false>(NG, grid, blk, s, aa);
}

pq_status attention_launches(const pq_ctx *ctx, const StepAppend *app, const StepWindow *win, int M, const void *q,
                             void *out, pq_dtype out_dtype,
                             uint8_t *k_codes, uint16_t *k_radii, uint8_t *v_codes, uint16_t *v_radii,
                             const int64_t *seq_start, const int32_t *ctx_len,
                             int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                             float softmax_scale, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !q || !out || !k_codes || !k_radii || !v_codes || !v_radii || !seq_start || !ctx_len || !workspace)
        return PQ_EINVAL;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || pool_tokens <= 0 || (pool_tokens & 63) || max_ctx < 0 || max_ctx > pool_tokens)
        return PQ_EINVAL;
    if (Hq % Hkv) return PQ_EINVAL;
    if (max_ctx > ((int64_t)1 << 26)) return PQ_EUNSUPPORTED; /* a sequence's tiles are addressed with 32-bit byte offsets */
    /* the work plan counts the tiles of all (sequence, kv head) streams in 31 bits (288 GB of cache hold 2^25) */
    if ((int64_t)B * Hkv * ((max_ctx + 63) / 64) >= ((int64_t)1 << 31) - 4096) return PQ_EUNSUPPORTED;
    if (out_dtype != PQ_BF16 && out_dtype != PQ_F32) return PQ_EINVAL;
    const int G = Hq / Hkv;
    if (M < 1 || M * G > 16) return PQ_EUNSUPPORTED;   /* at most 16 (query token, head) pairs per kv head */
    if ((app || win) && M != 1) return PQ_EUNSUPPORTED;
    const int NG = M * G <= 4 ? 1 : (M * G <= 8 ? 2 : 4);
    const bool deep = ctx->depth == 7;
    if (!pq_aligned16(q) || !pq_aligned16(out) || !pq_aligned16(k_codes) || !pq_aligned16(k_radii) ||
        !pq_aligned16(v_codes) || !pq_aligned16(v_radii) || !pq_aligned16(workspace))
        return PQ_EALIGN;
    if (app) {
        if (!app->xk || !app->xv || !app->dst_token) return PQ_EINVAL;
        if (app->xt != PQ_F32 && app->xt != PQ_BF16) return PQ_EINVAL;
        if (!pq_aligned16(app->xk) || !pq_aligned16(app->xv)) return PQ_EALIGN;
        if (2 * (int64_t)B * Hkv + (int64_t)B * Hq + 1 > 0x7FFFFFFF) return PQ_EINVAL;
    }
    if (win) {
        if (!win->win_k || !win->win_v || !win->win_len) return PQ_EINVAL;
        if (win->win_cap <= 0 || win->win_cap > 0x7FFFFFFF) return PQ_EINVAL;
        if (!pq_aligned16(win->win_k) || !pq_aligned16(win->win_v)) return PQ_EALIGN;
    }
    const Plan p = make_plan(B, Hq, Hkv, max_ctx, win ? win->win_cap : 0, M);
    if ((int64_t)B * Hkv * p.n_wchunks > 0x7FFFFFFF) return PQ_EINVAL;
    /* the partial kernel addresses the rotated queries and its partial results with 32-bit byte offsets */
    if ((uint64_t)B * M * Hq * (PQ_D * 2) > 0xFFFFFFFFull || p.o_bytes > 0xFFFFFFFFull) return PQ_EUNSUPPORTED;
    if (workspace_bytes < p.total) return PQ_ENOMEM;
    const PqDeviceState *ds = nullptr;
    pq_status st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    uint16_t *qrot = reinterpret_cast<uint16_t *>(ws);
    float *ws_ml = reinterpret_cast<float *>(ws + p.off_ml);
    float *ws_o = reinterpret_cast<float *>(ws + p.off_o);
    if ((int64_t)B * M * Hq >= 0x7FFFFFFF) return PQ_EINVAL; /* one more workgroup builds the plan */
    const int rows = B * M * Hq, row_blocks = (rows + kRotateRows - 1) / kRotateRows;

    int32_t *plan = reinterpret_cast<int32_t *>(ws + p.off_plan);
    const PlanArgs pa{seq_start, ctx_len, B, Hkv, max_ctx, pool_tokens / 64, p.slots, plan};
    RotateArgs ra{static_cast<const uint16_t *>(q), qrot, ds->S_f32, softmax_scale * kLog2e, ds->consts, ctx->hadamard};
    if (app) {
        AppendArgs ak{app->xk, k_codes, k_radii, pool_tokens / 64, pool_tokens, app->dst_token, Hkv, ds->S_f32, ds->consts, ctx->hadamard};
        AppendArgs av{app->xv, v_codes, v_radii, pool_tokens / 64, pool_tokens, app->dst_token, Hkv, ds->S_f32, ds->consts, ctx->hadamard};
        const int n = B * Hkv;
        const dim3 grid((unsigned)(2 * n + row_blocks + 1)), blk(512);
        if (app->xt == PQ_BF16) hipLaunchKernelGGL((pq_step_prologue_kernel<PQ_BF16>), grid, blk, 0, s, ra, ak, av, n, pa, rows, row_blocks);
        else hipLaunchKernelGGL((pq_step_prologue_kernel<PQ_F32>), grid, blk, 0, s, ra, ak, av, n, pa, rows, row_blocks);
    } else if (win) {
        WindowArgs wa{static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(win->win_k),
                      static_cast<const uint16_t *>(win->win_v), win->win_len, B, Hq, Hkv, (int)win->win_cap,
                      p.n_wchunks, softmax_scale * kLog2e, reinterpret_cast<float *>(ws + p.off_wml),
                      reinterpret_cast<float *>(ws + p.off_wo)};
        const int per_wave = (G >= 4 && G % 2 == 0) ? 2 : 1; /* query heads per wavefront (of one kv head's group) */
        const int64_t witems = (int64_t)B * (Hq / per_wave) * p.n_wchunks;
        const int64_t wblocks = (witems + kWindowWaves - 1) / kWindowWaves;
        if (wblocks + row_blocks + 1 > 0x7FFFFFFF) return PQ_EINVAL;
        const dim3 grid((unsigned)(row_blocks + 1 + wblocks)), blk(512);
        if (per_wave == 2) hipLaunchKernelGGL(pq_rotate_window_kernel<2>, grid, blk, 0, s, ra, pa, rows, row_blocks, wa, (int)wblocks);
        else hipLaunchKernelGGL(pq_rotate_window_kernel<1>, grid, blk, 0, s, ra, pa, rows, row_blocks, wa, (int)wblocks);
    } else {
        hipLaunchKernelGGL(pq_rotate_q_kernel, dim3((unsigned)row_blocks + 1u), dim3(512), 0, s, ra, pa, rows, row_blocks);
    }
    AttnArgs aa{};
    aa.qrot = qrot;
    aa.k_codes = k_codes; aa.v_codes = v_codes; aa.k_radii = k_radii; aa.v_radii = v_radii;
    aa.seq_start = seq_start; aa.ctx_len = ctx_len;
    aa.B = B; aa.Hq = Hq; aa.Hkv = Hkv; aa.M = M;
    aa.pool_tiles = pool_tokens / 64;
    aa.max_ctx = max_ctx;
    aa.plan = plan;
    aa.n_pieces = (int)p.pieces;
    aa.ws_ml = ws_ml; aa.ws_o = ws_o;
    aa.consts = ds->consts;
    aa.up_b5 = ctx->upper_bits[0]; aa.up_b6 = ctx->upper_bits[1]; aa.up_b7 = ctx->upper_bits[2];
    pq_prof_before(0, s);
    const dim3 grid(p.blocks), blk((unsigned)(waves_per_block(NG) * 64));
    launch_partial(NG, deep, grid, blk, s, aa);
    pq_prof_after(0, s);

    CombineArgs ca{ws_ml, ws_o, B, Hq, Hkv, M, plan,
                   ds->St_f32, out, out_dtype == PQ_F32 ? 1 : 0, ds->consts,
                   reinterpret_cast<const float *>(ws + p.off_wml), reinterpret_cast<const float *>(ws + p.off_wo),
                   win ? win->win_len : nullptr, p.n_wchunks, win ? (int)win->win_cap : 0, ctx->hadamard};
    if (win) hipLaunchKernelGGL(pq_attn_combine_kernel<true>, dim3(rows), dim3(512), 0, s, ca);
    else hipLaunchKernelGGL(pq_attn_combine_kernel<false>, dim3(rows), dim3(512), 0, s, ca);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

} // namespace

extern "C" pq_status pq_attn_decode_polar(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                          const uint8_t *k_codes, const uint16_t *k_radii,
                                          const uint8_t *v_codes, const uint16_t *v_radii,
                                          const int64_t *seq_start, const int32_t *ctx_len,
                                          int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                                          float softmax_scale, void *workspace, size_t workspace_bytes,
                                          void *hip_stream)
{
    /* the caches are only read on this path */
    return attention_launches(ctx, nullptr, nullptr, 1, q, out, out_dtype, const_cast<uint8_t *>(k_codes),
                              const_cast<uint16_t *>(k_radii), const_cast<uint8_t *>(v_codes),
                              const_cast<uint16_t *>(v_radii), seq_start, ctx_len, B, Hq, Hkv, pool_tokens, max_ctx,
                              softmax_scale, workspace, workspace_bytes, hip_stream);
}

/* ---- the entry point that allocates nothing ----
 * pq_attn_decode_polar with the workspace (rotated queries, work plan, partial results) in a
 * file-scope device array instead of a caller buffer.  `scratch` is the host-side stand-in of
 * the array: host code never passes it to a kernel or a copy, only the device address that
 * hipGetSymbolAddress returns for the current device (every device holds its own copy of the
 * array at its own address), resolved once per device and kept. */
static __device__ __align__(256) unsigned char scratch[PQ_STATIC_SCRATCH_BYTES];

namespace {
std::mutex g_scratch_mu;
void *g_scratch_ptr[PQ_MAX_DEVICES] = {nullptr};

pq_status scratch_of_current_device(void **out)
{
    int dev = -1;
    PQ_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= PQ_MAX_DEVICES) return PQ_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PQ_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PQ_OK;
}
} // namespace

extern "C" size_t pq_static_scratch_bytes(void) { return PQ_STATIC_SCRATCH_BYTES; }

extern "C" pq_status pq_prepare_device(const pq_ctx *ctx)
{
    if (!ctx) return PQ_EINVAL;
    const PqDeviceState *ds = nullptr;
    const pq_status st = pq_device_state(ctx, &ds); /* uploads the context's constants on first use (allocates) */
    if (st != PQ_OK) return st;
    void *p = nullptr;
    return scratch_of_current_device(&p);
}

extern "C" pq_status pq_attn_decode_polar_static(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                                 const uint8_t *k_codes, const uint16_t *k_radii,
                                                 const uint8_t *v_codes, const uint16_t *v_radii,
                                                 const int64_t *seq_start, const int32_t *ctx_len,
                                                 int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                                                 float softmax_scale, void *hip_stream)
{
    if (!ctx) return PQ_EINVAL;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || max_ctx < 0 || Hq % Hkv) return PQ_EINVAL;
    /* sizes first: a problem beyond the array is refused before anything else is looked at */
    if (max_ctx > ((int64_t)1 << 26) || (int64_t)B * Hkv * ((max_ctx + 63) / 64) >= ((int64_t)1 << 31) - 4096)
        return PQ_EUNSUPPORTED;
    if (make_plan(B, Hq, Hkv, max_ctx).total > (size_t)PQ_STATIC_SCRATCH_BYTES) return PQ_ESCRATCH;
    if (!pq_device_state_ready(ctx)) return PQ_ENOTREADY; /* the upload of the constants would allocate */
    void *ws = nullptr;
    const pq_status st = scratch_of_current_device(&ws);
    if (st != PQ_OK) return st;
    return attention_launches(ctx, nullptr, nullptr, 1, q, out, out_dtype, const_cast<uint8_t *>(k_codes),
                              const_cast<uint16_t *>(k_radii), const_cast<uint8_t *>(v_codes),
                              const_cast<uint16_t *>(v_radii), seq_start, ctx_len, B, Hq, Hkv, pool_tokens, max_ctx,
                              softmax_scale, ws, PQ_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" pq_status pq_decode_step_polar(const pq_ctx *ctx, const void *xk, const void *xv, pq_dtype xt,
                                          const int64_t *dst_token, const void *q, void *out, pq_dtype out_dtype,
                                          uint8_t *k_codes, uint16_t *k_radii, uint8_t *v_codes, uint16_t *v_radii,
                                          const int64_t *seq_start, const int32_t *ctx_len,
                                          int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                                          float softmax_scale, void *workspace, size_t workspace_bytes,
                                          void *hip_stream)
{
    const StepAppend app{xk, xv, xt, dst_token, Hkv};
    return attention_launches(ctx, &app, nullptr, 1, q, out, out_dtype, k_codes, k_radii, v_codes, v_radii, seq_start, ctx_len,
                              B, Hq, Hkv, pool_tokens, max_ctx, softmax_scale, workspace, workspace_bytes, hip_stream);
}

extern "C" pq_status pq_attn_decode_hybrid(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                           const uint8_t *k_codes, const uint16_t *k_radii,
                                           const uint8_t *v_codes, const uint16_t *v_radii,
                                           const int64_t *seq_start, const int32_t *ctx_len,
                                           const void *win_k, const void *win_v, const int32_t *win_len,
                                           int64_t win_cap, int B, int Hq, int Hkv, int64_t pool_tokens,
                                           int64_t max_ctx, float softmax_scale, void *workspace,
                                           size_t workspace_bytes, void *hip_stream)
{
    const StepWindow win{win_k, win_v, win_len, win_cap};
    return attention_launches(ctx, nullptr, &win, 1, q, out, out_dtype, const_cast<uint8_t *>(k_codes),
                              const_cast<uint16_t *>(k_radii), const_cast<uint8_t *>(v_codes),
                              const_cast<uint16_t *>(v_radii), seq_start, ctx_len, B, Hq, Hkv, pool_tokens, max_ctx,
                              softmax_scale, workspace, workspace_bytes, hip_stream);
}

extern "C" pq_status pq_attn_decode_polar_mq(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                             const uint8_t *k_codes, const uint16_t *k_radii,
                                             const uint8_t *v_codes, const uint16_t *v_radii,
                                             const int64_t *seq_start, const int32_t *ctx_len,
                                             int B, int M, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                                             float softmax_scale, void *workspace, size_t workspace_bytes,
                                             void *hip_stream)
{
    return attention_launches(ctx, nullptr, nullptr, M, q, out, out_dtype, const_cast<uint8_t *>(k_codes),
                              const_cast<uint16_t *>(k_radii), const_cast<uint8_t *>(v_codes),
                              const_cast<uint16_t *>(v_radii), seq_start, ctx_len, B, Hq, Hkv, pool_tokens, max_ctx,
                              softmax_scale, workspace, workspace_bytes, hip_stream);
}
