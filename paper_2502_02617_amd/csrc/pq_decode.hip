/*
 * pq_decode.hip -- pq_decode_kv (Algorithm 1, procedure DeQuant) and
 * pq_export_canonical (tile layout -> canonical records: 62 bytes, or 50 at
 * full recursion depth, where the block radii are themselves rebuilt from the
 * vector's radius and the codes of levels 7, 6, 5).
 *
 * DeQuant rebuilds each block top-down from its stored radius: at level l the
 * radius of node j splits into (r cos theta, r sin theta) with theta the
 * centroid selected by the node's code; after level 1 the 16 coordinates of
 * the block are known.  The optional trailing product with S^T is a 128x128
 * mat-vec per vector, done in fp32 with the rebuilt vector staged in LDS.
 * These kernels serve testing, export and fallback use; they read the tile
 * through the generic field accessors and are not tuned.
 */
#include "pq_common.h"

namespace {

constexpr int kTok = 16; /* tokens per workgroup */

struct DecodeArgs {
    const uint8_t *codes;
    const uint16_t *radii;
    int64_t pool_tiles;
    int64_t token0, n_tokens;
    int n_heads;
    void *out;
    int64_t ld_token, ld_head;
    int rotated;
    const PqDeviceConsts *consts;
    const float *St; /* St[j*128 + i] = S[i][j] */
    int deep;        /* recursion depth 7: the radius plane holds one word per token */
};

template <int KIND, int OT>
__global__ __launch_bounds__(128) void pq_decode_kernel(DecodeArgs a)
{
    __shared__ float sy[kTok][PQ_D];
    const int head = blockIdx.y;
    const int64_t t_base = (int64_t)blockIdx.x * kTok;
    const int tid = threadIdx.x;
    const PqDeviceConsts &K = *a.consts;
    {
        const int tl = tid >> 3, b = tid & 7; /* one thread per (token, block) */
        const int64_t t = t_base + tl;
        if (t < a.n_tokens) {
            const int64_t slot = a.token0 + t;
            const int64_t tile = slot >> 6;
            const int tau = (int)(slot & 63);
            const uint8_t *tc = a.codes + ((int64_t)head * a.pool_tiles + tile) * PQL_CODE_BYTES;
            const uint16_t *tr = a.radii + ((int64_t)head * a.pool_tiles + tile) * (a.deep ? PQ_DEEP_RADII_HALVES : PQL_RADII);
            PqBlockFields f = pql_read_block(KIND, tc, a.deep ? nullptr : tr, tau, b);
            float r4;
            if (a.deep)
                r4 = pq_deep_block_radius(reinterpret_cast<const uint32_t *>(tr)[tau], K.up_bits[0], K.up_bits[1], K.up_bits[2],
                                          reinterpret_cast<const float2 *>(&K.up_cs[0][0][0]), b);
            else
                r4 = (float)__builtin_bit_cast(_Float16, f.radius);
            float r3[2] = {r4 * K.cs234[2][f.c4][0], r4 * K.cs234[2][f.c4][1]};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t g6 = f.g6[h];
                uint32_t c2a = g6 >> 4, c3 = (g6 >> 2) & 3, c2b = g6 & 3;
                float r2a = r3[h] * K.cs234[1][c3][0], r2b = r3[h] * K.cs234[1][c3][1];
                float r1[4] = {r2a * K.cs234[0][c2a][0], r2a * K.cs234[0][c2a][1],
                               r2b * K.cs234[0][c2b][0], r2b * K.cs234[0][c2b][1]};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t c1 = (f.l1 >> (4 * (4 * h + q))) & 15;
                    sy[tl][16 * b + 8 * h + 2 * q] = r1[q] * K.cs1[c1][0];
                    sy[tl][16 * b + 8 * h + 2 * q + 1] = r1[q] * K.cs1[c1][1];
                }
            }
        }
    }
    __syncthreads();
    /* thread i produces output coordinate i of every token of the group */
    const int i = tid;
    float acc[kTok];
    if (a.rotated) {
#pragma unroll
        for (int t = 0; t < kTok; ++t) acc[t] = sy[t][i];
    } else {
#pragma unroll
        for (int t = 0; t < kTok; ++t) acc[t] = 0.0f;
        for (int j = 0; j < PQ_D; ++j) {
            float s = a.St[j * PQ_D + i]; /* S[i][j] */
#pragma unroll
            for (int t = 0; t < kTok; ++t) acc[t] += sy[t][j] * s;
        }
    }
#pragma unroll
    for (int t = 0; t < kTok; ++t) {
        int64_t tt = t_base + t;
        if (tt >= a.n_tokens) break;
        int64_t at = tt * a.ld_token + (int64_t)head * a.ld_head + i;
        if (OT == PQ_F32) static_cast<float *>(a.out)[at] = acc[t];
        else {
            uint32_t u = __float_as_uint(acc[t]);
            uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
            static_cast<uint16_t *>(a.out)[at] = (uint16_t)r;
        }
    }
}

struct ExportArgs {
    const uint8_t *codes;
    const uint16_t *radii;
    int64_t pool_tiles;
    int64_t token0, n_tokens;
    uint8_t *rec;
    int deep;
};

/* one thread per (token, block): writes the block's share of the canonical record */
template <int KIND>
__global__ __launch_bounds__(256) void pq_export_kernel(ExportArgs a)
{
    const int head = blockIdx.y;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t t = idx >> 3;
    const int b = (int)(idx & 7);
    if (t >= a.n_tokens) return;
    const int64_t slot = a.token0 + t;
    const int64_t tile = slot >> 6;
    const int tau = (int)(slot & 63);
    const uint8_t *tc = a.codes + ((int64_t)head * a.pool_tiles + tile) * PQL_CODE_BYTES;
    const uint16_t *tr = a.radii + ((int64_t)head * a.pool_tiles + tile) * (a.deep ? PQ_DEEP_RADII_HALVES : PQL_RADII);
    PqBlockFields f = pql_read_block(KIND, tc, a.deep ? nullptr : tr, tau, b);
    uint8_t *rec = a.rec + ((int64_t)head * a.n_tokens + t) * (a.deep ? PQ_DEEP_RECORD_BYTES : PQ_RECORD_BYTES);
    /* level 1: pairs 8b..8b+7 -> bytes 4b..4b+3, earlier code in the high nibble */
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t c_even = (f.l1 >> (8 * k)) & 15, c_odd = (f.l1 >> (8 * k + 4)) & 15;
        rec[4 * b + k] = (uint8_t)((c_even << 4) | c_odd);
    }
    /* level 2: nodes 4b..4b+3 -> byte 32 + b, earlier code in the higher bits */
    uint32_t c2_0 = f.g6[0] >> 4, c2_1 = f.g6[0] & 3, c2_2 = f.g6[1] >> 4, c2_3 = f.g6[1] & 3;
    rec[32 + b] = (uint8_t)((c2_0 << 6) | (c2_1 << 4) | (c2_2 << 2) | c2_3);
    uint32_t c3_0 = (f.g6[0] >> 2) & 3, c3_1 = (f.g6[1] >> 2) & 3;
    /* level 3 (2 codes) and level 4 (1 code) share bytes with the neighbouring
       blocks: gather them across the 8 lanes that hold one token's blocks */
    uint32_t nib3 = (c3_0 << 2) | c3_1; /* 4 bits of byte 40 + b/2 */
    uint32_t other3 = __shfl_xor(nib3, 1);
    if ((b & 1) == 0) rec[40 + (b >> 1)] = (uint8_t)((nib3 << 4) | other3);
    uint32_t acc4 = f.c4 << (6 - 2 * (b & 3)); /* 2 bits of byte 44 + b/4 */
    acc4 |= __shfl_xor(acc4, 1);
    acc4 |= __shfl_xor(acc4, 2);
    if ((b & 3) == 0) rec[44 + (b >> 2)] = (uint8_t)acc4;
    if (a.deep) {
        if (b == 0) { /* code word of levels 5..7, then the vector's radius, both little endian */
            const uint32_t word = reinterpret_cast<const uint32_t *>(tr)[tau];
            rec[46] = (uint8_t)(word & 0xFF);
            rec[47] = (uint8_t)((word >> 8) & 0xFF);
            rec[48] = (uint8_t)((word >> 16) & 0xFF);
            rec[49] = (uint8_t)(word >> 24);
        }
    } else {
        rec[46 + 2 * b] = (uint8_t)(f.radius & 0xFF);
        rec[47 + 2 * b] = (uint8_t)(f.radius >> 8);
    }
}

} // namespace

extern "C" pq_status pq_decode_kv(const pq_ctx *ctx, pq_kind kind, const uint8_t *codes, const uint16_t *radii,
                                  int64_t pool_tokens, int64_t token0, int64_t n_tokens, int n_heads,
                                  void *out, pq_dtype ot, int64_t ld_token, int64_t ld_head,
                                  int rotated, void *hip_stream)
{
    if (!ctx || !codes || !radii || !out) return PQ_EINVAL;
    if (kind != PQ_KEY && kind != PQ_VALUE) return PQ_EINVAL;
    if (ot != PQ_F32 && ot != PQ_BF16) return PQ_EINVAL;
    if (n_tokens < 0 || n_heads <= 0 || n_heads > 65535 || pool_tokens <= 0 || (pool_tokens & 63) || token0 < 0) return PQ_EINVAL;
    if (token0 + n_tokens > pool_tokens || ld_token < 0 || ld_head < 0) return PQ_EINVAL;
    if (!pq_aligned16(codes) || !pq_aligned16(radii) || !pq_aligned16(out)) return PQ_EALIGN;
    if (n_tokens == 0) return PQ_OK;
    const PqDeviceState *ds = nullptr;
    pq_status st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    DecodeArgs a{codes, radii, pool_tokens / 64, token0, n_tokens, n_heads, out, ld_token, ld_head, rotated,
                 ds->consts, ds->St_f32, ctx->depth == 7 ? 1 : 0};
    dim3 grid((unsigned)((n_tokens + kTok - 1) / kTok), (unsigned)n_heads), block(128);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (kind == PQ_KEY) {
        if (ot == PQ_F32) hipLaunchKernelGGL((pq_decode_kernel<PQ_KEY, PQ_F32>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((pq_decode_kernel<PQ_KEY, PQ_BF16>), grid, block, 0, s, a);
    } else {
        if (ot == PQ_F32) hipLaunchKernelGGL((pq_decode_kernel<PQ_VALUE, PQ_F32>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((pq_decode_kernel<PQ_VALUE, PQ_BF16>), grid, block, 0, s, a);
    }
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

extern "C" pq_status pq_export_canonical(const pq_ctx *ctx, pq_kind kind, const uint8_t *codes,
                                         const uint16_t *radii, int64_t pool_tokens, int64_t token0,
                                         int64_t n_tokens, int n_heads, uint8_t *rec, void *hip_stream)
{
    if (!ctx || !codes || !radii || !rec) return PQ_EINVAL;
    if (kind != PQ_KEY && kind != PQ_VALUE) return PQ_EINVAL;
    if (n_tokens < 0 || n_heads <= 0 || n_heads > 65535 || pool_tokens <= 0 || (pool_tokens & 63) || token0 < 0) return PQ_EINVAL;
    if (token0 + n_tokens > pool_tokens) return PQ_EINVAL;
    if (!pq_aligned16(codes) || !pq_aligned16(radii)) return PQ_EALIGN;
    if (n_tokens == 0) return PQ_OK;
    ExportArgs a{codes, radii, pool_tokens / 64, token0, n_tokens, rec, ctx->depth == 7 ? 1 : 0};
    dim3 grid((unsigned)((n_tokens * 8 + 255) / 256), (unsigned)n_heads), block(256);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (kind == PQ_KEY) hipLaunchKernelGGL((pq_export_kernel<PQ_KEY>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((pq_export_kernel<PQ_VALUE>), grid, block, 0, s, a);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}
