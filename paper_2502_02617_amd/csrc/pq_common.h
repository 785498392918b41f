/*
 * pq_common.h -- shared declarations of libpolarquant's translation units:
 * the context object, the device-side constant block and launch helpers.
 */
#ifndef PQ_COMMON_H
#define PQ_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/polarquant.h"
#include "pq_layout.h"

/* Lookup tables of the attention kernels as the host builds them (dwords); the kernel spreads the small ones
 * over a column per lane when it copies them into LDS.
 *   TQ  [1024][2]: quarter table, by the stored quarter index Q = c1' << 6 | c2 << 4 | c1: the four binary16 products
 *                  (cos t2 cos t1, cos t2 sin t1, sin t2 cos t1', sin t2 sin t1') -- the level-2 x level-1 part of
 *                  the four coordinates of a quarter.  Values multiply an entry by the quarter's radius.
 *   TQA [64]:      its first pair alone, by Q & 63 = c2 << 4 | c1; TQB [64]: its second pair, by Q >> 4 = c1' << 2 | c2.
 *                  Keys fetch the two and use them as a matrix-core operand as they are.
 *   TBF [64][4]:   block table for the keys, by the stored block index B = c4 << 4 | c3 << 2 | c3': the four fp32
 *                  products (cos t4 cos t3, cos t4 sin t3, sin t4 cos t3', sin t4 sin t3') -- what the block radius
 *                  is multiplied by to give the radii of its four quarters.
 *   TBH [64][2]:   the same as binary16 pairs for the values: dword 0 the first half-block's two, dword 1 the second's.
 *   UP  [3][8][2]: full-depth recursion: fp32 (cos, sin) of the centroids of levels 5, 6, 7. */
enum {
    PQ_TAB_TQ = 0, PQ_TAB_TQA = 2048, PQ_TAB_TQB = 2112, PQ_TAB_TBF = 2176, PQ_TAB_TBH = 2432, PQ_TAB_UP = 2560,
    PQ_TAB_DWORDS = 2608
};

/* Constants every kernel reads; one copy per device in global memory. */
struct PqDeviceConsts {
    /* Quantisation by comparison in the tangent domain (Algorithm 1, Quant):
       an angle psi = atan(v/u), u, v >= 0, lies above the inner boundary t iff
       v > tan(t) * u.  tan_b[l-1] = {tan t_1, tan t_2, tan t_3} of level l
       within one quadrant (level 1: boundaries pi/8, pi/4, 3pi/8). */
    float tan_b[4][4];
    /* cos / sin of the centroids, fp32 (DeQuant). */
    float cs1[16][2];
    float cs234[3][4][2];
    /* Codebooks other than the analytic ones (set with pq_set_codebooks): general != 0.
       Level 1 is then quantised through the pseudo-angle p(psi) in [0, 4) -- quadrant number
       plus |y| / (|x| + |y|) or |x| / (|x| + |y|), monotone in psi -- and a table over 512
       equal cells of p: cell c holds the number of level-1 boundaries in the cells before it
       and the pseudo-angle of the one boundary inside it (+inf if none); code = count +
       (p > that).  Levels 2-4 use tan_b with all three of its entries. */
    int general;
    struct Lut1Cell { float thr; uint32_t count; } lut1[512];
    /* Full-depth recursion (depth == 7, Definition 1): levels 5, 6, 7 join the 8 block radii of a
       vector with 4 + 2 + 1 more angles of up_bits[l-5] bits each; the vector keeps one radius.
       up_tan2[l-5][k]: squared tangent of inner boundary k of level l (the recursion carries
       squared radii); up_cs[l-5][c]: (cos, sin) of centroid c.  depth == 4: unused. */
    int depth;
    int up_bits[3];
    float up_tan2[3][7];
    float up_cs[3][8][2];
    /* The attention kernels' LDS table block, entry for entry (layout: PQ_TAB_* above), copied by a
       workgroup in 16-byte pieces. */
    alignas(16) uint32_t attn_tab[PQ_TAB_DWORDS];
};

/* Radius plane of a tile.  Depth 4: 512 binary16 block radii (pq_layout.h).  Depth 7: 64 words,
   word tau = (binary16 radius of the vector << 16) | code word of levels 5..7 (level-5 codes
   j = 0..3 at bits [j b5, (j+1) b5), level-6 codes j = 0, 1 at 4 b5 + j b6, level 7 at
   4 b5 + 2 b6), the same for key and value tiles. */
#define PQ_DEEP_RADII_HALVES 128
#define PQ_DEEP_RECORD_BYTES 50

/* Per-device constant buffers of a context (created on first use). */
struct PqDeviceState {
    bool ready = false;
    PqDeviceConsts *consts = nullptr; /* device */
    float *S_f32 = nullptr;           /* device [128][128], S[i][j]              */
    float *St_f32 = nullptr;          /* device [128][128], St[j][i] = S[i][j]   */
    uint16_t *S_bf16x3 = nullptr;     /* device: three bf16 terms of S (of sqrt(d) * S if its entries are all
                                         +-1/sqrt(d): one term, the others zero) in MFMA operand order */
};

#define PQ_MAX_DEVICES 16

/* S = D H / sqrt(128) with H the Sylvester Hadamard matrix H[i][j] = (-1)^popcount(i & j) and D a diagonal of
   signs (a randomised Hadamard preconditioner, Section 1): the products of single vectors with S and S^T -- query
   rotation, the appended key and value, the un-rotation of the output -- then run as a fast Walsh-Hadamard
   transform inside one wavefront (7 x 64 additions) instead of 128 x 128 products against a matrix read from
   memory.  Passed to the kernels by value. */
struct PqHadamard {
    uint32_t on;     /* 0: S is a general matrix */
    uint32_t neg[4]; /* bit i set: D_i = -1 */
};

struct pq_ctx {
    int d;
    uint64_t seed;
    double S[PQ_D * PQ_D];
    /* every entry of S is +-1/sqrt(d) (a sign-flipped Hadamard matrix, say): sqrt(d) * S is then
       exact in bf16 and the encode kernel multiplies by one term instead of three */
    bool unit_entries;
    PqHadamard hadamard;    /* on: S is D H / sqrt(d) exactly (found by comparing the entries) */
    bool general_codebooks; /* codebooks replaced by pq_set_codebooks */
    double centroids[4][16];
    double boundaries[4][17];
    int depth;              /* 4, or 7 after pq_set_recursion_depth */
    int upper_bits[3];      /* bits of levels 5, 6, 7 (depth 7) */
    double upper_centroids[3][8];
    double upper_boundaries[3][9];
    PqDeviceConsts host_consts;
    std::mutex mu;
    PqDeviceState dev[PQ_MAX_DEVICES];
};

/* Returns the constant buffers of the current device, uploading them on the
 * first call per device.  PQ_EHIP if there is no usable device. */
pq_status pq_device_state(const pq_ctx *ctx, const PqDeviceState **out);
/* true once pq_device_state has uploaded the constants of ctx to the current device */
bool pq_device_state_ready(const pq_ctx *ctx);

#define PQ_HIP_TRY(expr)                         \
    do {                                         \
        hipError_t e__ = (expr);                 \
        if (e__ != hipSuccess) return PQ_EHIP;   \
    } while (0)

/* Optional timing of the two dominant kernels with HIP events on the caller's
 * stream (see pq_profile_begin / pq_profile_end).  kind: 0 attention partial
 * kernel, 1 encode kernel.  No-ops unless profiling is on. */
void pq_prof_before(int kind, hipStream_t s);
void pq_prof_after(int kind, hipStream_t s);

/* Lloyd-Max quantiser of Lemma 2's density of level `level` (>= 2) with K cells: centroids[K], boundaries[K + 1] */
void pq_lloyd_max(int level, int K, double *centroids, double *boundaries);

static inline bool pq_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

/* ---- small dense products with S: one vector per 512-thread workgroup ----
 * out[j] = sum_k in[k] * M[k*128 + j].  Thread (kq, j) accumulates the k-quarter kq with
 * all 32 loads in flight at once (these kernels are latency bound, not bandwidth bound);
 * the four quarter sums are added in a fixed order by the threads of quarter 0.
 * The matrix part does not depend on the vector: a kernel requests it first
 * (matrix_slice_load) and overlaps its latency with fetching the vector. */
struct MatrixSlice {
    float m[32];
};

static __device__ __forceinline__ void matrix_slice_load(MatrixSlice &s, const float *M, int tid)
{
    const int kq = tid >> 7, j = tid & 127;
#pragma unroll
    for (int k = 0; k < 32; ++k) s.m[k] = M[(32 * kq + k) * PQ_D + j];
}

static __device__ __forceinline__ float vector_times_slice(const float (&sin)[PQ_D], const MatrixSlice &s,
                                                           float (&spart)[4][PQ_D], int tid)
{
    const int kq = tid >> 7, j = tid & 127;
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fmaf(sin[32 * kq + k], s.m[k], acc);
    spart[kq][j] = acc;
    __syncthreads();
    return ((spart[0][j] + spart[1][j]) + spart[2][j]) + spart[3][j];
}

#if defined(__HIPCC__)
/* ---- fast Walsh-Hadamard transform of 128 values in one wavefront ----
 * Lane l holds elements l (lo) and l + 64 (hi); on return it holds elements l and l + 64 of
 * w_j = sum_i v_i (-1)^popcount(i & j), unscaled: one butterfly stage inside the lane, six across lanes. */
static __device__ __forceinline__ void pq_fwht128(float &lo, float &hi, int lane)
{
    const float a = lo + hi, b = lo - hi;
    lo = a;
    hi = b;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float pl = __shfl_xor(lo, d), ph = __shfl_xor(hi, d);
        lo = (lane & d) ? pl - lo : lo + pl;
        hi = (lane & d) ? ph - hi : hi + ph;
    }
}

static __device__ __forceinline__ float pq_hadamard_sign(const PqHadamard &h, int i)
{
    return ((h.neg[i >> 5] >> (i & 31)) & 1u) ? -1.0f : 1.0f;
}

#define PQ_INV_SQRT_D 0.08838834764831845f /* 1 / sqrt(128) */

/* ---- depth 7: block radii from a tile's radius-plane word (DeQuant's levels 7, 6, 5) ----
 * cs: the (cos, sin) pairs of the centroids, [3][8] (levels 5, 6, 7), in LDS or global memory.
 * Products in fp32, in the order radius * level 7 * level 6 * level 5. */
static __device__ __forceinline__ float pq_half_bits_to_float(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

static __device__ __forceinline__ void pq_deep_block_radii(uint32_t word, int b5, int b6, int b7, const float2 *cs,
                                                           float (&r)[8])
{
    const float R = pq_half_bits_to_float(word >> 16);
    const float2 t7 = cs[16 + __builtin_amdgcn_ubfe(word, 4 * b5 + 2 * b6, b7)];
    const float r6[2] = {R * t7.x, R * t7.y};
    float r5[4];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float2 t6 = cs[8 + __builtin_amdgcn_ubfe(word, 4 * b5 + j * b6, b6)];
        r5[2 * j] = r6[j] * t6.x;
        r5[2 * j + 1] = r6[j] * t6.y;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 t5 = cs[__builtin_amdgcn_ubfe(word, j * b5, b5)];
        r[2 * j] = r5[j] * t5.x;
        r[2 * j + 1] = r5[j] * t5.y;
    }
}

/* the same for one block b (same products, same order) */
static __device__ __forceinline__ float pq_deep_block_radius(uint32_t word, int b5, int b6, int b7, const float2 *cs, int b)
{
    const float R = pq_half_bits_to_float(word >> 16);
    const float2 t7 = cs[16 + __builtin_amdgcn_ubfe(word, 4 * b5 + 2 * b6, b7)];
    const float2 t6 = cs[8 + __builtin_amdgcn_ubfe(word, 4 * b5 + (b >> 2) * b6, b6)];
    const float2 t5 = cs[__builtin_amdgcn_ubfe(word, (b >> 1) * b5, b5)];
    const float r6 = R * ((b & 4) ? t7.y : t7.x);
    const float r5 = r6 * ((b & 2) ? t6.y : t6.x);
    return r5 * ((b & 1) ? t5.y : t5.x);
}

/* Procedure Quant above level 4: the number of inner boundaries below atan(sqrt(v2 / u2)), from
 * squared radii; boundary k is passed when v2 > tan^2(t_k) u2 (one rounding in the fused form). */
static __device__ __forceinline__ uint32_t pq_quant_upper(float u2, float v2, const float *tan2, int n_bounds)
{
    uint32_t c = 0;
#pragma unroll
    for (int k = 0; k < 7; ++k)
        if (k < n_bounds) c += (__builtin_fmaf(tan2[k], u2, -v2) < 0.0f) ? 1u : 0u;
    return c;
}
#endif

/* Layout of S_bf16x3 (halves): [term 3][row-tile 4][k-step 8][lane 64][8].
 * Lane l = 32*kg + i of (term, rt, ks) holds S_term[64*kg + 8*ks + e][col(rt, i)]
 * for e = 0..7, where the 32 rows of row-tile rt map to rotated coordinates
 * col(rt, i) = 16*(4*((i>>2)&1) + rt) + 4*(i>>3) + (i&3). */
#define PQ_SB_TERM_STRIDE (4 * 8 * 64 * 8)

#endif
