/*
 * pq_encode.hip -- pq_encode_kv / pq_encode_kv_pair / pq_append_kv: Algorithm 1
 * lines 2 and 4 (precondition with S, procedure Polar, procedure Quant) plus
 * bit-packing into the tile layout, for gfx950.
 *
 * Bulk kernel (pq_encode_kv, and for keys and values in one launch
 * pq_encode_kv_pair; the append kernel lives in pq_polar.h):
 * one wavefront owns one destination tile (64 token slots of one head plane).
 *   1. y = x * S on the matrix cores.  S is held as three bf16 terms
 *      S1 + S2 + S3 (24 significant bits) so that bf16 MFMAs with fp32
 *      accumulation reproduce an fp32-accurate rotation; bf16 inputs are
 *      exact operands, fp32 inputs are split the same way (x1 + x2 + x3) and
 *      the six products above 2^-24 are accumulated.
 *      The product is computed transposed, D = S^T-tile (32 rotated
 *      coordinates) x X^T (32 vectors), with the rows of each S^T tile
 *      ordered so that a lane ends up with complete blocks of 16 consecutive
 *      rotated coordinates of one vector in its accumulator registers: the
 *      whole polar recursion of a block is then register-local.
 *   2. Four polar levels per block; every angle is quantised by comparing
 *      in the tangent domain (v > tan(t) * u for each inner boundary t, on
 *      squared radii above level 1), which is the nearest-centroid rule of
 *      procedure Quant without evaluating an arctangent or, but for the
 *      block radius, a square root.
 *   3. The fields are assembled into whole dwords in registers (full tiles) or
 *      scattered with LDS atomics (partially written tiles) into an image of
 *      the tile in LDS, and the image is written out with full-width stores.
 *   At recursion depth 7 the recursion goes on over the block radii of a vector
 *   (levels 5, 6, 7) and one word per token replaces the block radii.
 */
#include "pq_common.h"
#include "pq_polar.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

/* wavefronts per workgroup (two per SIMD: the kernel uses the whole register file).  Sixteen
   wavefronts working on one 32-vector half at a time in 128 registers measured slower: every
   A-operand fetch then feeds one matrix instruction instead of two. */
template <int XT> struct EncodeShape { static constexpr int waves = 8; };
/* tile image in LDS: the code bytes, then the radius plane (512 binary16 block radii, or at
   depth 7 the 64 words of radius and upper-level codes) */
template <bool DEEP> struct TileImage {
    static constexpr int radii_halves = DEEP ? PQ_DEEP_RADII_HALVES : PQL_RADII;
    static constexpr int dwords = (PQL_CODE_BYTES + radii_halves * 2) / 4; /* 992 or 800 */
};

struct EncodeArgs {
    const void *x;
    int64_t ld_token, ld_head;
    uint8_t *codes;
    uint16_t *radii;
    int64_t pool_tiles;
    int64_t pool_tokens;
    /* tokens [dst0, dst0 + n) of every head plane */
    int64_t dst0, n_tokens;
    int64_t first_tile, n_tiles; /* tiles spanned by the range */
    int n_heads;
    int64_t n_items;
    const uint4 *S_bf16x3;
    const PqDeviceConsts *consts;
};

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ uint32_t bf16_rne_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

union BOperand {
    bf16x8 v;
    uint4 q;
    uint32_t w[4];
};

/* Scatter the fields of block b of slot tau into the tile image (codes, then radii), without branches: every
 * field is shifted to its place inside a pair of dwords and OR-ed in.  The image is shared by the lanes of one
 * wavefront and the fields of different slots share dwords: LDS atomics.  CLEAR = false: the image started as
 * zeros (a tile written whole); CLEAR = true: it holds the tile's present contents and the field's bits are
 * cleared first.  The positions are those of pq_layout.h, written out per plane. */
template <bool CLEAR>
__device__ __forceinline__ void put_pair(uint32_t *img, uint32_t at0, uint32_t at1, uint32_t field, uint32_t width, uint32_t sh)
{
    if (CLEAR) {
        const uint64_t m = (uint64_t)((1u << width) - 1u) << sh;
        atomicAnd(&img[at0], ~(uint32_t)m);
        atomicAnd(&img[at1], ~(uint32_t)(m >> 32));
    }
    const uint64_t w = (uint64_t)field << sh;
    atomicOr(&img[at0], (uint32_t)w);
    atomicOr(&img[at1], (uint32_t)(w >> 32));
}

template <int KIND, bool CLEAR, bool DEEP>
__device__ __forceinline__ void emit_block(uint32_t *img, int tau, int b, const BlockCodes &bc)
{
    const uint32_t q0 = bc.q[0], q1 = bc.q[1], q2 = bc.q[2], q3 = bc.q[3], bi = bc.bi;
    uint32_t radius_half;
    if (KIND == PQ_KEY) {
        /* dword d of the token's string: planes of 4, 4, 3 dwords per token, then one half per token */
        auto at = [&](uint32_t d) {
            return d < 4u ? 4u * tau + d : d < 8u ? (PQL_OFF_P1 / 4 - 4) + 4u * tau + d
                 : d < 11u ? (PQL_OFF_P2 / 4 - 8) + 3u * tau + d : PQL_OFF_KP3 / 4 + ((uint32_t)tau >> 1);
        };
        const uint32_t bit = PQL_BLOCK_BITS * (uint32_t)b, d = bit >> 5, sh = bit & 31u;
        /* the string's last half sits in a dword shared by two tokens */
        const uint32_t sh1 = (d + 1u == 11u) ? 16u * ((uint32_t)tau & 1u) : 0u;
        /* 46 bits reach into a third dword when they start above bit 18 (never in the string's last dwords) */
        const bool third = sh > 18u;
        const uint32_t a0 = at(d), a1 = at(d + 1u), a2 = at(third ? d + 2u : d);
        if (CLEAR) {
            const uint64_t m = ((1ull << PQL_BLOCK_BITS) - 1ull) << sh;
            atomicAnd(&img[a0], ~(uint32_t)m);
            atomicAnd(&img[a1], ~((uint32_t)(m >> 32) << sh1));
            if (third) atomicAnd(&img[a2], ~(0x3FFFu >> (32u - sh)));
        }
        const uint32_t lo = q0 | (q1 << 10) | (q2 << 20) | (q3 << 30), hi = (q3 >> 2) | (bi << 8); /* 32 + 14 bits */
        const uint64_t w = (((uint64_t)hi << 32) | lo) << sh;
        atomicOr(&img[a0], (uint32_t)w);
        atomicOr(&img[a1], (uint32_t)(w >> 32) << sh1);
        if (third) atomicOr(&img[a2], hi >> (32u - sh));
        radius_half = 8u * tau + b;
    } else {
        const uint32_t i = (uint32_t)tau >> 4, g = ((uint32_t)tau >> 2) & 3u, e = (uint32_t)tau & 3u, s = 4u * i + e;
        /* dword d of lane lam's string: planes of 4, 4, 2 dwords per lane */
        auto at = [&](uint32_t lam, uint32_t d) {
            return d < 4u ? 4u * lam + d : d < 8u ? (PQL_OFF_P1 / 4 - 4) + 4u * lam + d : (PQL_OFF_P2 / 4 - 8) + 2u * lam + d;
        };
        const uint32_t bit = PQL_SLOT_BITS * s, d = bit >> 5, sh = bit & 31u;
        /* the dword after a string's last one belongs to the next lane (or the next plane): it gets zeros */
        const uint32_t lam0 = 16u * g + 2u * b;
        put_pair<CLEAR>(img, at(lam0, d), at(lam0, d + 1u), q0 | (q1 << 10), PQL_SLOT_BITS, sh);
        put_pair<CLEAR>(img, at(lam0 + 1u, d), at(lam0 + 1u, d + 1u), q2 | (q3 << 10), PQL_SLOT_BITS, sh);
        const uint32_t bbit = 6u * s, base = PQL_OFF_VB / 4 + 3u * (8u * g + b) + (bbit >> 5);
        put_pair<CLEAR>(img, base, base + 1u, bi, 6u, bbit & 31u);
        radius_half = 16u * (8u * g + b) + s;
    }
    if (!DEEP) reinterpret_cast<uint16_t *>(img)[PQL_CODE_BYTES / 2 + radius_half] = bc.radius;
}

/* lanes 0..31: the value of lane + 32; lanes 32..63: the value of lane - 32 */
__device__ __forceinline__ uint32_t from_other_half(uint32_t x, int upper_half)
{
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return upper_half ? r[0] : r[1];
}

/* NTERMS = 3: S as three bf16 terms.  NTERMS = 1: every entry of S is +-1/sqrt(128), the
   operand is sqrt(128) * S (exactly +-1 in bf16), one product per k-step replaces three and
   the common factor is taken out of the block radius (the angles do not see it). */
/* GENERAL: codebooks set by the caller; level 1 goes through the pseudo-angle cell table (staged
   in LDS), the upper levels compare against three free boundaries. */
/* DEEP: recursion to level 7.  The squared radii of a vector's blocks are kept as the row tiles
   complete (a lane half holds blocks 4H..4H+3 of its vectors); levels 5 and 6 then run inside the
   lane, level 7 joins the two halves with one lane exchange, and the vector's radius and upper
   codes go into its word of the radius plane. */
/* LDS of the encode kernels, shared by all their variants (a workgroup runs alone on its CU):
   S in A-operand order, 32 KB per bf16 term; one tile image per wavefront; the level-1 cell table of
   caller-set codebooks. */
__shared__ uint4 sS[3 * 4 * 8 * 64];
__shared__ __align__(16) uint32_t sImg[8][TileImage<false>::dwords];
__shared__ PqDeviceConsts::Lut1Cell sLut[512];

/* The tiles of one launch share: workgroup `block` of `n_blocks` takes every n_blocks-th group of
   eight items (an item = one destination tile of one head plane). */
template <int XT, int KIND, int NTERMS, bool GENERAL, bool DEEP>
__device__ __forceinline__ void encode_tiles(const EncodeArgs &a, int block, int n_blocks)
{
    constexpr int kImgDwords = TileImage<DEEP>::dwords, kRadiiHalves = TileImage<DEEP>::radii_halves;
    constexpr int kWaves = EncodeShape<XT>::waves, kThreads = kWaves * 64;
    static_assert(kWaves == 8, "sImg holds eight tile images");
    constexpr int kSChunks = NTERMS * 4 * 8 * 64;   /* 16-byte chunks of the copy of S that is used */

    const int lane = threadIdx.x & 63;
    /* same value in all lanes: keeps the item geometry and the tile pointers in scalar registers */
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 31, H = lane >> 5; /* vector within the 32-vector group, lane half */

    /* bf16 input: both 32-vector halves of the tile share every A-operand fetch (halves the
       LDS traffic); fp32 input carries three bf16 terms per value and goes one half at a time */
    constexpr int NXT = (XT == PQ_BF16) ? 1 : 3; /* bf16 terms of x */
    constexpr int NVT = (XT == PQ_BF16) ? 2 : 1; /* 32-vector halves per pass */
    /* bf16 input: the operand registers of a tile are dead once its last row tile has been multiplied,
       so the next tile's rows are requested then, under the last quantisation stage, and the first
       tile's before S is staged */
    constexpr bool kPipelined = (XT == PQ_BF16);
    BOperand xb[NVT][NXT][8];

    /* which tile and which source rows an item covers */
    struct Geometry {
        int head;
        int64_t tile;       /* tile index inside the head plane */
        int tau_lo, tau_hi; /* slots [tau_lo, tau_hi) of the tile are written */
        int64_t src_t0;     /* source token index of slot tau_lo */
    };
    /* Item = head * n_tiles + tile.  The 64-bit division happens once per wavefront; from then on the position
       advances by the (head, tile) parts of the stride between a wavefront's items. */
    struct Position {
        int head;
        int64_t tile_in; /* tile within the range, below n_tiles */
    };
    const int64_t item_stride = (int64_t)n_blocks * (EncodeShape<XT>::waves);
    const int64_t item0 = (int64_t)block * (EncodeShape<XT>::waves) + wave;
    const int stride_heads = (int)(item_stride / a.n_tiles);
    const int64_t stride_tiles = item_stride % a.n_tiles;
    auto advance = [&](Position p) {
        p.head += stride_heads;
        p.tile_in += stride_tiles;
        if (p.tile_in >= a.n_tiles) {
            p.tile_in -= a.n_tiles;
            ++p.head;
        }
        return p;
    };
    auto geometry = [&](const Position &p) {
        Geometry g;
        g.head = p.head;
        g.tile = a.first_tile + p.tile_in;
        const int64_t lo = g.tile * 64 > a.dst0 ? g.tile * 64 : a.dst0;
        const int64_t hi = (g.tile + 1) * 64 < a.dst0 + a.n_tokens ? (g.tile + 1) * 64 : a.dst0 + a.n_tokens;
        g.tau_lo = (int)(lo - g.tile * 64);
        g.tau_hi = (int)(hi - g.tile * 64);
        g.src_t0 = lo - a.dst0;
        return g;
    };
    /* element offset of the input row that feeds slot tau_ of the item; a lane without a slot
       to write reads the first row of the range again: its results are never emitted, and
       every address stays inside the input */
    auto source_row = [&](const Geometry &g, int tau_) {
        const bool ok = tau_ >= g.tau_lo && tau_ < g.tau_hi;
        const int64_t t_src = g.src_t0 + (ok ? tau_ - g.tau_lo : 0);
        return t_src * a.ld_token + (int64_t)g.head * a.ld_head;
    };
    /* B operands of a bf16 tile: this lane's 8-coordinate slices of its two vectors, every k-step
       (coordinates 64 H + 8 ks .. + 7: one contiguous half row per lane) */
    auto load_bf16_rows = [&](const Geometry &g) {
        if constexpr (XT == PQ_BF16) {
#pragma unroll
            for (int v = 0; v < NVT; ++v) {
                const int64_t row = source_row(g, 32 * v + j);
                const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.x) + row);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) xb[v][0][ks].q = xr[8 * H + ks];
            }
        }
    };
    Position pos{(int)(item0 / a.n_tiles), item0 % a.n_tiles};
    if (kPipelined && item0 < a.n_items) load_bf16_rows(geometry(pos));

    {   /* all of a thread's chunks are requested before the first one is stored: one round trip to L2
           instead of one per chunk */
        constexpr int kPerThread = kSChunks / kThreads;
        static_assert(kSChunks % kThreads == 0, "S chunks must divide evenly over the workgroup");
        uint4 stage[kPerThread];
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) stage[i] = a.S_bf16x3[threadIdx.x + i * kThreads];
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) sS[threadIdx.x + i * kThreads] = stage[i];
    }
    __syncthreads();

    Thresholds th = load_thresholds(*a.consts, NTERMS == 1 ? 0.08838834764831845f /* 1/sqrt(128) */ : 1.0f);
    if (GENERAL) {
        for (int c = threadIdx.x; c < 512; c += kThreads) sLut[c] = a.consts->lut1[c];
        th.lut1 = sLut;
        __syncthreads();
    }

    UpperTables ut = {};
    if (DEEP) ut = load_upper_tables(*a.consts);

    uint32_t *img = sImg[wave];

    /* The hardware prefers the older of the two wavefronts of a SIMD, which then finishes well before the other
       and leaves it to run alone; each wavefront lowers its issue priority as it works through its items, so
       that the one behind catches up. */
    const int my_items = item0 < a.n_items ? (int)((a.n_items - item0 + item_stride - 1) / item_stride) : 0;
    int items_done = 0;
    for (int64_t item = item0; item < a.n_items; item += item_stride, pos = advance(pos)) {
        {
            const int q4 = 4 * items_done; /* prio = 3 - floor(4 items_done / my_items) */
            const int prio = 3 - (q4 >= my_items) - (q4 >= 2 * my_items) - (q4 >= 3 * my_items);
            if (prio >= 3) __builtin_amdgcn_s_setprio(3);
            else if (prio == 2) __builtin_amdgcn_s_setprio(2);
            else if (prio == 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
            ++items_done;
        }
        const Geometry geo = geometry(pos);
        const int head = geo.head, tau_lo = geo.tau_lo, tau_hi = geo.tau_hi;
        const int64_t tile = geo.tile;
        const bool full = (tau_lo == 0 && tau_hi == 64);
        uint8_t *gcodes = a.codes + ((int64_t)head * a.pool_tiles + tile) * PQL_CODE_BYTES;
        uint16_t *gradii = a.radii + ((int64_t)head * a.pool_tiles + tile) * kRadiiHalves;

        /* ---- tile image: zeros, or the tile's present contents if only part of it is written ---- */
        if (full) {
            for (int c = lane; c < kImgDwords / 4; c += 64) reinterpret_cast<uint4 *>(img)[c] = make_uint4(0u, 0u, 0u, 0u);
        } else {
            const uint32_t *gc = reinterpret_cast<const uint32_t *>(gcodes);
            const uint32_t *gr = reinterpret_cast<const uint32_t *>(gradii);
            for (int c = lane; c < PQL_CODE_BYTES / 4; c += 64) img[c] = gc[c];
            for (int c = lane; c < kRadiiHalves / 2; c += 64) img[PQL_CODE_BYTES / 4 + c] = gr[c];
        }
        wave_lds_sync();

        for (int vt0 = 0; vt0 < 2; vt0 += NVT) {
            /* wave-uniform skip of a pass with nothing to write */
            if (32 * (vt0 + NVT) <= tau_lo || 32 * vt0 >= tau_hi) continue;

            bool valid[NVT];
            int tau[NVT];
#pragma unroll
            for (int v = 0; v < NVT; ++v) {
                tau[v] = 32 * (vt0 + v) + j;
                valid[v] = tau[v] >= tau_lo && tau[v] < tau_hi;
                /* ---- B operands: this lane's 8-coordinate slices of its vector, every k-step
                   (coordinates 64 H + 8 ks .. + 7: one contiguous half row per lane) ---- */
                if constexpr (XT != PQ_BF16) { /* bf16 rows were requested ahead (load_bf16_rows) */
                    const int64_t row = source_row(geo, tau[v]);
                    const float4 *xr = reinterpret_cast<const float4 *>(static_cast<const float *>(a.x) + row);
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        float f[8];
                        const float4 p0 = xr[16 * H + 2 * ks], p1 = xr[16 * H + 2 * ks + 1]; /* coordinates 64 H + 8 ks .. + 7 */
                        f[0] = p0.x; f[1] = p0.y; f[2] = p0.z; f[3] = p0.w;
                        f[4] = p1.x; f[5] = p1.y; f[6] = p1.z; f[7] = p1.w;
#pragma unroll
                        for (int e = 0; e < 8; e += 2) {
                            uint32_t w1[2], w2[2], w3[2];
#pragma unroll
                            for (int z = 0; z < 2; ++z) {
                                float val = f[e + z];
                                uint32_t b1 = bf16_rne_bits(val);
                                float r1 = val - __uint_as_float(b1 << 16);
                                uint32_t b2 = bf16_rne_bits(r1);
                                float r2 = r1 - __uint_as_float(b2 << 16);
                                uint32_t b3 = bf16_rne_bits(r2);
                                w1[z] = b1; w2[z] = b2; w3[z] = b3;
                            }
                            xb[v][0][ks].w[e / 2] = w1[0] | (w1[1] << 16);
                            xb[v][NXT > 1 ? 1 : 0][ks].w[e / 2] = w2[0] | (w2[1] << 16);
                            xb[v][NXT > 2 ? 2 : 0][ks].w[e / 2] = w3[0] | (w3[1] << 16);
                        }
                    }
                }
            }

            /* D[i][j] = sum_k S[k][col(rt,i)] * x[j][k]: 32 rotated coordinates x 32 vectors per row
               tile rt.  The products of row tile rt+1 are issued between the steps of the polar
               recursion of row tile rt, in a fixed interleaving: each pair of matrix instructions
               is followed by a slice of vector work that does not depend on them, so the matrix
               cores run while the vector ALU quantises.  Stage -1 only multiplies, stage 3 only
               quantises. */
            f32x16 acc_even[NVT], acc_odd[NVT];
            float q4[NVT][4]; /* DEEP: squared radii of blocks 4H .. 4H+3 */
#pragma unroll
            for (int st = -1; st < 4; ++st) {
                f32x16 (&cur)[NVT] = (st & 1) ? acc_odd : acc_even;   /* row tile st: quantised now */
                f32x16 (&nxt)[NVT] = (st & 1) ? acc_even : acc_odd;   /* row tile st+1: accumulated now */
                const bool mul = st < 3, quant = st >= 0;
                if (kPipelined && st == 3 && item + item_stride < a.n_items) load_bf16_rows(geometry(advance(pos)));
                PolarState ps[NVT];
                BOperand sa_next;
                if (mul) sa_next.q = sS[(((NTERMS - 1) * 4 + (st + 1)) * 8 + 0) * 64 + lane];
                /* The vector work that goes with k-step ks comes in U units (level-1 pair ks in two parts
                   and the upper-level nodes it completes, per vector); they are spread evenly behind the
                   NM matrix instructions of the k-step. */
                constexpr int NM = NXT == 1 ? NVT * NTERMS : NVT * (NTERMS == 3 ? 6 : 3);
                constexpr int U = 3 * NVT;
                auto unit = [&](int ks, int u) {
                    const int v = NVT == 2 ? (u < 4 ? u >> 1 : u - 4) : 0;
                    const int part = NVT == 2 ? (u < 4 ? (u & 1) : 2) : u;
                    if (part == 0) polar_level1_a<GENERAL>(ps[v], cur[v], ks, th);
                    if (part == 1) polar_level1_b<GENERAL>(ps[v], cur[v], ks);
                    if (part == 2) polar_upper<GENERAL>(ps[v], ks, th);
                };
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    int m = 0;
#pragma unroll
                    for (int term = NTERMS - 1; term >= 0; --term) { /* smallest terms first */
                        if (mul) {
                            /* A operand of this step; the next one is requested from LDS right away */
                            const BOperand sa = sa_next;
                            const int nterm = term > 0 ? term - 1 : NTERMS - 1, nks = term > 0 ? ks : ks + 1;
                            if (nks < 8) sa_next.q = sS[((nterm * 4 + (st + 1)) * 8 + nks) * 64 + lane];
#pragma unroll
                            for (int v = 0; v < NVT; ++v)
#pragma unroll
                                for (int xt = 0; xt < NXT; ++xt) {
                                    if (xt + term > 2) continue; /* below 2^-24 of the leading product */
                                    /* the first product of a row tile starts from a zero accumulator operand */
                                    const bool first = (ks == 0 && term == NTERMS - 1 && xt == 0);
                                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                                    nxt[v] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa.v, xb[v][xt][ks].v, first ? zero : nxt[v], 0, 0, 0);
                                    if (quant) {
#pragma unroll
                                        for (int u = m * U / NM; u < (m + 1) * U / NM; ++u) unit(ks, u);
                                        __builtin_amdgcn_sched_barrier(0);
                                    }
                                    ++m;
                                }
                        }
                    }
                    if (!mul) {
#pragma unroll
                        for (int u = 0; u < U; ++u) unit(ks, u);
                    }
                }
                if (quant) {
                    /* lane (H, j): cur[v][r] = rotated coordinate 16*(4H + st) + r of vector tau[v] */
                    const int b = 4 * H + st;
                    if (DEEP) {
#pragma unroll
                        for (int v = 0; v < NVT; ++v) q4[v][st < 0 ? 0 : st] = ps[v].out.q4;
                    }
                    /* a full tile has a slot for every lane: no per-lane branch there.  (Around a
                       single vector's fields it would let the optimiser move that vector's whole
                       recursion behind the branch and undo the interleaving above.) */
                    if (full) {
#pragma unroll
                        for (int v = 0; v < NVT; ++v) emit_block<KIND, false, DEEP>(img, tau[v], b, ps[v].out);
                    } else {
#pragma unroll
                        for (int v = 0; v < NVT; ++v)
                            if (valid[v]) emit_block<KIND, true, DEEP>(img, tau[v], b, ps[v].out);
                    }
                }
            }
            if (DEEP) {
#pragma unroll
                for (int v = 0; v < NVT; ++v) {
                    const UpperHalf mine = polar_upper_half(q4[v], H, ut);
                    UpperHalf other;
                    other.codes = from_other_half(mine.codes, H);
                    other.q6 = __uint_as_float(from_other_half(__float_as_uint(mine.q6), H));
                    const uint32_t word = H == 0 ? polar_upper_join(mine, other, th.radius_scale, ut)
                                                 : polar_upper_join(other, mine, th.radius_scale, ut);
                    if (H == 0 && valid[v]) img[PQL_CODE_BYTES / 4 + tau[v]] = word;
                }
            }
        }
        wave_lds_sync();

        /* ---- image -> global, 16 bytes per lane per store ---- */
        {
            const uint4 *src = reinterpret_cast<const uint4 *>(img);
            uint4 *dc = reinterpret_cast<uint4 *>(gcodes);
            uint4 *dr = reinterpret_cast<uint4 *>(gradii);
            for (int c = lane; c < PQL_CODE_BYTES / 16; c += 64) dc[c] = src[c];
            for (int c = lane; c < kRadiiHalves * 2 / 16; c += 64) dr[c] = src[PQL_CODE_BYTES / 16 + c];
        }
        wave_lds_sync();
    }
}

template <int XT, int KIND, int NTERMS, bool GENERAL, bool DEEP>
__global__ __launch_bounds__(EncodeShape<XT>::waves * 64) void pq_encode_kernel(EncodeArgs a)
{
    encode_tiles<XT, KIND, NTERMS, GENERAL, DEEP>(a, (int)blockIdx.x, (int)gridDim.x);
}

/* Keys and values of the same tokens in one launch: workgroups [0, k_blocks) encode the key tiles, the
   rest the value tiles.  One launch instead of two, S staged once per CU, twice as many tiles per
   wavefront to spread the start-up over. */
template <int XT, int NTERMS, bool GENERAL, bool DEEP>
__global__ __launch_bounds__(EncodeShape<XT>::waves * 64) void pq_encode_pair_kernel(EncodeArgs k, EncodeArgs v, int k_blocks)
{
    if ((int)blockIdx.x < k_blocks) encode_tiles<XT, PQ_KEY, NTERMS, GENERAL, DEEP>(k, (int)blockIdx.x, k_blocks);
    else encode_tiles<XT, PQ_VALUE, NTERMS, GENERAL, DEEP>(v, (int)blockIdx.x - k_blocks, (int)gridDim.x - k_blocks);
}

template <int XT, int KIND>
__global__ __launch_bounds__(512) void pq_append_kernel(AppendArgs a)
{
    append_vector<XT>(a, KIND, (int)blockIdx.x);
}

/* keys and values of the same tokens in one launch: workgroups [0, n) take the key vectors,
   [n, 2n) the value vectors (a decode step appends both; one launch saves a dispatch) */
template <int XT>
__global__ __launch_bounds__(512) void pq_append_pair_kernel(AppendArgs k, AppendArgs v, int n)
{
    if ((int)blockIdx.x < n) append_vector<XT>(k, PQ_KEY, (int)blockIdx.x);
    else append_vector<XT>(v, PQ_VALUE, (int)blockIdx.x - n);
}

template <int XT, int KIND, int NTERMS, bool GENERAL, bool DEEP>
pq_status launch_encode(const EncodeArgs &a, hipStream_t stream)
{
    static int cached_cus[PQ_MAX_DEVICES] = {0};
    int dev = 0;
    PQ_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= PQ_MAX_DEVICES) return PQ_EUNSUPPORTED;
    if (cached_cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached_cus[dev] = n;
    }
    const int cus = cached_cus[dev];
    constexpr int kWaves = EncodeShape<XT>::waves, kThreads = kWaves * 64;
    int64_t blocks = (a.n_items + kWaves - 1) / kWaves;
    if (blocks > cus) blocks = cus;
    if (blocks < 1) blocks = 1;
    pq_prof_before(1, stream);
    hipLaunchKernelGGL((pq_encode_kernel<XT, KIND, NTERMS, GENERAL, DEEP>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, a);
    pq_prof_after(1, stream);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

template <int XT, int NTERMS, bool GENERAL, bool DEEP>
pq_status launch_encode_pair(const EncodeArgs &k, const EncodeArgs &v, hipStream_t stream)
{
    int dev = 0, cus = 0;
    PQ_HIP_TRY(hipGetDevice(&dev));
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    constexpr int kWaves = EncodeShape<XT>::waves, kThreads = kWaves * 64;
    /* both streams have the same number of items: half of the CUs each, at least one workgroup */
    int64_t per_kind = (k.n_items + kWaves - 1) / kWaves;
    if (per_kind > cus / 2) per_kind = cus / 2;
    if (per_kind < 1) per_kind = 1;
    pq_prof_before(1, stream);
    hipLaunchKernelGGL((pq_encode_pair_kernel<XT, NTERMS, GENERAL, DEEP>), dim3((unsigned)(2 * per_kind)), dim3(kThreads), 0,
                       stream, k, v, (int)per_kind);
    pq_prof_after(1, stream);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

template <int NTERMS, bool GENERAL, bool DEEP>
pq_status dispatch_pair_terms(const EncodeArgs &k, const EncodeArgs &v, pq_dtype xt, hipStream_t stream)
{
    return xt == PQ_BF16 ? launch_encode_pair<PQ_BF16, NTERMS, GENERAL, DEEP>(k, v, stream)
                         : launch_encode_pair<PQ_F32, NTERMS, GENERAL, DEEP>(k, v, stream);
}

pq_status dispatch_encode_pair(const EncodeArgs &k, const EncodeArgs &v, pq_dtype xt, bool unit_entries, bool general,
                               bool deep, hipStream_t stream)
{
    if (deep) {
        if (general)
            return unit_entries ? dispatch_pair_terms<1, true, true>(k, v, xt, stream) : dispatch_pair_terms<3, true, true>(k, v, xt, stream);
        return unit_entries ? dispatch_pair_terms<1, false, true>(k, v, xt, stream) : dispatch_pair_terms<3, false, true>(k, v, xt, stream);
    }
    if (general)
        return unit_entries ? dispatch_pair_terms<1, true, false>(k, v, xt, stream) : dispatch_pair_terms<3, true, false>(k, v, xt, stream);
    return unit_entries ? dispatch_pair_terms<1, false, false>(k, v, xt, stream) : dispatch_pair_terms<3, false, false>(k, v, xt, stream);
}

template <int NTERMS, bool GENERAL, bool DEEP>
pq_status dispatch_encode_terms(const EncodeArgs &a, pq_dtype xt, pq_kind kind, hipStream_t stream)
{
    if (xt == PQ_BF16)
        return kind == PQ_KEY ? launch_encode<PQ_BF16, PQ_KEY, NTERMS, GENERAL, DEEP>(a, stream)
                              : launch_encode<PQ_BF16, PQ_VALUE, NTERMS, GENERAL, DEEP>(a, stream);
    return kind == PQ_KEY ? launch_encode<PQ_F32, PQ_KEY, NTERMS, GENERAL, DEEP>(a, stream)
                          : launch_encode<PQ_F32, PQ_VALUE, NTERMS, GENERAL, DEEP>(a, stream);
}

pq_status dispatch_encode(const EncodeArgs &a, pq_dtype xt, pq_kind kind, bool unit_entries, bool general, bool deep,
                          hipStream_t stream)
{
    if (deep) {
        if (general)
            return unit_entries ? dispatch_encode_terms<1, true, true>(a, xt, kind, stream)
                                : dispatch_encode_terms<3, true, true>(a, xt, kind, stream);
        return unit_entries ? dispatch_encode_terms<1, false, true>(a, xt, kind, stream)
                            : dispatch_encode_terms<3, false, true>(a, xt, kind, stream);
    }
    if (general)
        return unit_entries ? dispatch_encode_terms<1, true, false>(a, xt, kind, stream)
                            : dispatch_encode_terms<3, true, false>(a, xt, kind, stream);
    return unit_entries ? dispatch_encode_terms<1, false, false>(a, xt, kind, stream)
                        : dispatch_encode_terms<3, false, false>(a, xt, kind, stream);
}

} // namespace

extern "C" const char *pq_kernel_name_encode(void) { return "pq_encode_kernel"; }

namespace {

/* argument checks and launch geometry shared by pq_encode_kv and pq_encode_kv_pair */
pq_status make_encode_args(const void *x, pq_dtype xt, int64_t n_tokens, int n_heads, int64_t ld_token, int64_t ld_head,
                           uint8_t *codes, uint16_t *radii, int64_t pool_tokens, int64_t dst_token0, EncodeArgs &a)
{
    if (!x || !codes || !radii) return PQ_EINVAL;
    if (n_tokens < 0 || n_heads <= 0 || pool_tokens <= 0 || (pool_tokens & 63) || dst_token0 < 0) return PQ_EINVAL;
    if (dst_token0 + n_tokens > pool_tokens) return PQ_EINVAL;
    if (ld_token < 0 || ld_head < 0) return PQ_EINVAL;
    const int64_t elems16 = xt == PQ_BF16 ? 8 : 4;
    if (!pq_aligned16(x) || !pq_aligned16(codes) || !pq_aligned16(radii)) return PQ_EALIGN;
    if ((ld_token % elems16) || (ld_head % elems16)) return PQ_EALIGN;
    a = EncodeArgs{};
    a.x = x; a.ld_token = ld_token; a.ld_head = ld_head;
    a.codes = codes; a.radii = radii; a.pool_tiles = pool_tokens / 64; a.pool_tokens = pool_tokens;
    a.dst0 = dst_token0; a.n_tokens = n_tokens;
    a.first_tile = dst_token0 / 64;
    a.n_tiles = (dst_token0 + n_tokens + 63) / 64 - a.first_tile;
    a.n_heads = n_heads;
    a.n_items = a.n_tiles * n_heads;
    return PQ_OK;
}

void set_device_tables(EncodeArgs &a, const PqDeviceState *ds)
{
    a.S_bf16x3 = reinterpret_cast<const uint4 *>(ds->S_bf16x3);
    a.consts = ds->consts;
}

} // namespace

extern "C" pq_status pq_encode_kv(const pq_ctx *ctx, const void *x, pq_dtype xt, pq_kind kind,
                                  int64_t n_tokens, int n_heads, int64_t ld_token, int64_t ld_head,
                                  uint8_t *codes, uint16_t *radii, int64_t pool_tokens,
                                  int64_t dst_token0, void *hip_stream)
{
    if (!ctx) return PQ_EINVAL;
    if (n_tokens == 0) return PQ_OK;
    if (xt != PQ_F32 && xt != PQ_BF16) return PQ_EINVAL;
    if (kind != PQ_KEY && kind != PQ_VALUE) return PQ_EINVAL;
    EncodeArgs a;
    pq_status st = make_encode_args(x, xt, n_tokens, n_heads, ld_token, ld_head, codes, radii, pool_tokens, dst_token0, a);
    if (st != PQ_OK) return st;
    const PqDeviceState *ds = nullptr;
    st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    set_device_tables(a, ds);
    return dispatch_encode(a, xt, kind, ctx->unit_entries, ctx->general_codebooks, ctx->depth == 7,
                           static_cast<hipStream_t>(hip_stream));
}

extern "C" pq_status pq_encode_kv_pair(const pq_ctx *ctx, const void *xk, const void *xv, pq_dtype xt,
                                       int64_t n_tokens, int n_heads, int64_t ld_token, int64_t ld_head,
                                       uint8_t *k_codes, uint16_t *k_radii, uint8_t *v_codes, uint16_t *v_radii,
                                       int64_t pool_tokens, int64_t dst_token0, void *hip_stream)
{
    if (!ctx) return PQ_EINVAL;
    if (n_tokens == 0) return PQ_OK;
    if (xt != PQ_F32 && xt != PQ_BF16) return PQ_EINVAL;
    EncodeArgs ak, av;
    pq_status st = make_encode_args(xk, xt, n_tokens, n_heads, ld_token, ld_head, k_codes, k_radii, pool_tokens, dst_token0, ak);
    if (st != PQ_OK) return st;
    st = make_encode_args(xv, xt, n_tokens, n_heads, ld_token, ld_head, v_codes, v_radii, pool_tokens, dst_token0, av);
    if (st != PQ_OK) return st;
    const PqDeviceState *ds = nullptr;
    st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    set_device_tables(ak, ds);
    set_device_tables(av, ds);
    return dispatch_encode_pair(ak, av, xt, ctx->unit_entries, ctx->general_codebooks, ctx->depth == 7,
                                static_cast<hipStream_t>(hip_stream));
}

extern "C" pq_status pq_append_kv(const pq_ctx *ctx, const void *x, pq_dtype xt, pq_kind kind,
                                  int n_seq, int n_heads, uint8_t *codes, uint16_t *radii,
                                  int64_t pool_tokens, const int64_t *dst_token, void *hip_stream)
{
    if (!ctx) return PQ_EINVAL;
    if (n_seq == 0) return PQ_OK;
    if (!x || !codes || !radii || !dst_token) return PQ_EINVAL;
    if (xt != PQ_F32 && xt != PQ_BF16) return PQ_EINVAL;
    if (kind != PQ_KEY && kind != PQ_VALUE) return PQ_EINVAL;
    if (n_seq < 0 || n_heads <= 0 || pool_tokens <= 0 || (pool_tokens & 63)) return PQ_EINVAL;
    if ((int64_t)n_seq * n_heads > 0x7FFFFFFF) return PQ_EINVAL;
    if (!pq_aligned16(x) || !pq_aligned16(codes) || !pq_aligned16(radii)) return PQ_EALIGN;
    const PqDeviceState *ds = nullptr;
    pq_status st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    AppendArgs a{x, codes, radii, pool_tokens / 64, pool_tokens, dst_token, n_heads, ds->S_f32, ds->consts, ctx->hadamard};
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    dim3 grid((unsigned)(n_seq * n_heads)), block(512);
    if (xt == PQ_BF16) {
        if (kind == PQ_KEY) hipLaunchKernelGGL((pq_append_kernel<PQ_BF16, PQ_KEY>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((pq_append_kernel<PQ_BF16, PQ_VALUE>), grid, block, 0, s, a);
    } else {
        if (kind == PQ_KEY) hipLaunchKernelGGL((pq_append_kernel<PQ_F32, PQ_KEY>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((pq_append_kernel<PQ_F32, PQ_VALUE>), grid, block, 0, s, a);
    }
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

extern "C" pq_status pq_append_kv_pair(const pq_ctx *ctx, const void *xk, const void *xv, pq_dtype xt,
                                       int n_seq, int n_heads, uint8_t *k_codes, uint16_t *k_radii,
                                       uint8_t *v_codes, uint16_t *v_radii, int64_t pool_tokens,
                                       const int64_t *dst_token, void *hip_stream)
{
    if (!ctx) return PQ_EINVAL;
    if (n_seq == 0) return PQ_OK;
    if (!xk || !xv || !k_codes || !k_radii || !v_codes || !v_radii || !dst_token) return PQ_EINVAL;
    if (xt != PQ_F32 && xt != PQ_BF16) return PQ_EINVAL;
    if (n_seq < 0 || n_heads <= 0 || pool_tokens <= 0 || (pool_tokens & 63)) return PQ_EINVAL;
    if (2 * (int64_t)n_seq * n_heads > 0x7FFFFFFF) return PQ_EINVAL;
    if (!pq_aligned16(xk) || !pq_aligned16(xv) || !pq_aligned16(k_codes) || !pq_aligned16(k_radii) ||
        !pq_aligned16(v_codes) || !pq_aligned16(v_radii)) return PQ_EALIGN;
    const PqDeviceState *ds = nullptr;
    pq_status st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    AppendArgs ak{xk, k_codes, k_radii, pool_tokens / 64, pool_tokens, dst_token, n_heads, ds->S_f32, ds->consts, ctx->hadamard};
    AppendArgs av{xv, v_codes, v_radii, pool_tokens / 64, pool_tokens, dst_token, n_heads, ds->S_f32, ds->consts, ctx->hadamard};
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int n = n_seq * n_heads;
    dim3 grid((unsigned)(2 * n)), block(512);
    if (xt == PQ_BF16) hipLaunchKernelGGL((pq_append_pair_kernel<PQ_BF16>), grid, block, 0, s, ak, av, n);
    else hipLaunchKernelGGL((pq_append_pair_kernel<PQ_F32>), grid, block, 0, s, ak, av, n);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}
