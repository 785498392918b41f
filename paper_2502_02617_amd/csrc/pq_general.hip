/*
 * pq_general.hip -- the general PolarQuant format: any recursion depth from 4 to 7
 * and other bit widths than Section 4.1's (Definition 1 recurses to log2 d; the
 * remark after Theorem 1 leaves the codebook size of each level free).
 *
 * This is the plain path next to the tuned one: records are kept one after
 * another in the canonical general layout (all codes of level 1, then level 2,
 * ..., in one little-endian bit stream padded to a byte, then the 128 >> depth
 * binary16 radii), every field goes through a generic bit reader, and the
 * kernels are simple fp32 code, one wavefront per vector or per (sequence,
 * query head):
 *   encode     y = x S (fp32 sums in index order), procedure Polar level by
 *              level in LDS, procedure Quant as a count of the cell boundaries
 *              (midpoints of neighbouring centroids) below the angle
 *   decode     procedure DeQuant: centroid cos/sin products from the top level
 *              down, then the trailing S^T
 *   attention  Eq. 5 in the rotated domain: q' = q S once, every cached token
 *              dequantised without its S^T, online softmax, one S^T at the end
 * Section 4.1's own configuration (depth 4, bits 4/2/2/2) and its depth-7
 * extension have the tuned kernels of pq_encode.hip / pq_attn.hip; this file
 * accepts them too (same numbers, other layout), which is how it is tested
 * against them.
 */
#include "pq_common.h"

#include <cmath>
#include <cstring>

namespace {

constexpr int kGenMaxCells = 16;
constexpr int kGenMaxRecord = 96; /* bytes: depth 4 with bits 4/3/3/3 needs 53 + 16 */

struct GenFormat {
    int depth;
    int bits[7];
    int level_off[7];  /* first angle of level l inside the level-major numbering */
    int code_bytes, rec_bytes, n_radii;
    float bound[7][kGenMaxCells - 1]; /* inner cell boundaries */
    float cosv[7][kGenMaxCells], sinv[7][kGenMaxCells];
};

bool general_format_ok(const pq_general_format *f)
{
    if (!f || f->depth < 4 || f->depth > 7) return false;
    if (f->bits[0] != 3 && f->bits[0] != 4) return false;
    for (int l = 1; l < 4; ++l)
        if (f->bits[l] != 2 && f->bits[l] != 3) return false;
    for (int l = 4; l < f->depth; ++l)
        if (f->bits[l] < 1 || f->bits[l] > 3) return false;
    return true;
}

int general_code_bits(const pq_general_format *f)
{
    int n = 0;
    for (int l = 0; l < f->depth; ++l) n += (PQ_D >> (l + 1)) * f->bits[l];
    return n;
}

pq_status make_format(const pq_general_format *f, const double *cbg, GenFormat *g)
{
    if (!general_format_ok(f) || !cbg) return PQ_EINVAL;
    memset(g, 0, sizeof(*g));
    g->depth = f->depth;
    int off = 0, cboff = 0;
    const double half_pi = 1.57079632679489661923, two_pi = 6.28318530717958647692;
    for (int l = 0; l < f->depth; ++l) {
        const int K = 1 << f->bits[l];
        g->bits[l] = f->bits[l];
        g->level_off[l] = off;
        off += PQ_D >> (l + 1);
        for (int k = 0; k < K; ++k) {
            const double c = cbg[cboff + k];
            if (!std::isfinite(c) || c < 0.0 || c > (l == 0 ? two_pi : half_pi)) return PQ_EINVAL;
            if (k > 0 && !(c > cbg[cboff + k - 1])) return PQ_EINVAL;
            g->cosv[l][k] = (float)cos(c);
            g->sinv[l][k] = (float)sin(c);
            if (k > 0) g->bound[l][k - 1] = (float)(0.5 * (c + cbg[cboff + k - 1]));
        }
        cboff += K;
    }
    g->code_bytes = (general_code_bits(f) + 7) / 8;
    g->n_radii = PQ_D >> f->depth;
    g->rec_bytes = g->code_bytes + 2 * g->n_radii;
    return PQ_OK;
}

__device__ __forceinline__ uint32_t gen_get_bits(const uint8_t *stream, int pos, int width)
{
    uint32_t v = stream[pos >> 3] | ((uint32_t)stream[(pos >> 3) + 1] << 8); /* width <= 4: two bytes suffice */
    return (v >> (pos & 7)) & ((1u << width) - 1u);
}

__device__ __forceinline__ uint16_t gen_radius_bits(float r)
{
    return __builtin_bit_cast(uint16_t, (_Float16)fminf(r, 65504.f)); /* saturates at the largest finite binary16 */
}

/* position of angle j of level l in the record's bit stream */
__device__ __forceinline__ int gen_bit_pos(const GenFormat &f, int l, int j)
{
    int pos = 0;
    for (int m = 0; m < l; ++m) pos += (PQ_D >> (m + 1)) * f.bits[m];
    return pos + j * f.bits[l];
}

/* ---- encode: one wavefront per vector ---- */
template <int XT>
__global__ __launch_bounds__(64) void pq_general_encode_kernel(GenFormat f, const void *x, int64_t ld_vector, int64_t n,
                                                               const float *S, uint8_t *rec)
{
    __shared__ float sx[PQ_D];
    __shared__ float buf[2][PQ_D];
    __shared__ uint32_t srec[kGenMaxRecord / 4];
    const int64_t v = blockIdx.x;
    const int tid = threadIdx.x;
    if (v >= n) return;
    for (int c = tid; c < PQ_D; c += 64) {
        const int64_t at = v * ld_vector + c;
        sx[c] = XT == PQ_BF16 ? __uint_as_float((uint32_t)static_cast<const uint16_t *>(x)[at] << 16)
                              : static_cast<const float *>(x)[at];
    }
    for (int c = tid; c < kGenMaxRecord / 4; c += 64) srec[c] = 0u;
    __syncthreads();
    {   /* y_j = sum_i x_i S[i][j], i ascending; this thread's two columns */
        float a0 = 0.f, a1 = 0.f;
        for (int i = 0; i < PQ_D; ++i) {
            const float2 s2 = *reinterpret_cast<const float2 *>(S + i * PQ_D + 2 * tid);
            a0 = fmaf(sx[i], s2.x, a0);
            a1 = fmaf(sx[i], s2.y, a1);
        }
        buf[0][2 * tid] = a0;
        buf[0][2 * tid + 1] = a1;
    }
    __syncthreads();
    int cur = 0;
    for (int l = 0; l < f.depth; ++l) {
        const int n_ang = PQ_D >> (l + 1), K = 1 << f.bits[l];
        if (tid < n_ang) {
            const float a = buf[cur][2 * tid], b = buf[cur][2 * tid + 1];
            float ang = atan2f(b, a);
            if (l == 0 && ang < 0.f) ang += 6.28318530717958647692f;
            uint32_t code = 0;
            for (int k = 0; k < K - 1; ++k) code += ang > f.bound[l][k] ? 1u : 0u; /* nearest centroid, ties to the lower cell */
            const int pos = gen_bit_pos(f, l, tid);
            atomicOr(&srec[pos >> 5], code << (pos & 31));
            if ((pos & 31) + f.bits[l] > 32) atomicOr(&srec[(pos >> 5) + 1], code >> (32 - (pos & 31)));
            buf[cur ^ 1][tid] = sqrtf(a * a + b * b);
        }
        cur ^= 1;
        __syncthreads();
    }
    uint8_t *out = rec + v * f.rec_bytes;
    const uint8_t *img = reinterpret_cast<const uint8_t *>(srec);
    for (int c = tid; c < f.code_bytes; c += 64) out[c] = img[c];
    if (tid < f.n_radii) {
        const uint16_t h = gen_radius_bits(buf[cur][tid]);
        out[f.code_bytes + 2 * tid] = (uint8_t)(h & 0xFF);
        out[f.code_bytes + 2 * tid + 1] = (uint8_t)(h >> 8);
    }
}

/* orders the LDS accesses of the lanes of one wavefront (the buffers below belong to a single wavefront) */
__device__ __forceinline__ void gen_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

/* DeQuant's loops for one record by one wavefront (lane = 0..63): r^(0) (rotated domain) into
   buf[returned index][0..127]; buf is the wavefront's own */
__device__ __forceinline__ int gen_dequant_rotated(const GenFormat &f, const uint8_t *rec, float (&buf)[2][PQ_D], int lane)
{
    int cur = 0;
    if (lane < f.n_radii) {
        const uint16_t h = (uint16_t)(rec[f.code_bytes + 2 * lane] | (rec[f.code_bytes + 2 * lane + 1] << 8));
        buf[0][lane] = (float)__builtin_bit_cast(_Float16, h);
    }
    gen_wave_sync();
    for (int l = f.depth - 1; l >= 0; --l) {
        const int n_ang = PQ_D >> (l + 1);
        if (lane < n_ang) {
            const uint32_t code = gen_get_bits(rec, gen_bit_pos(f, l, lane), f.bits[l]);
            const float r = buf[cur][lane];
            buf[cur ^ 1][2 * lane] = r * f.cosv[l][code];
            buf[cur ^ 1][2 * lane + 1] = r * f.sinv[l][code];
        }
        cur ^= 1;
        gen_wave_sync();
    }
    return cur;
}

/* ---- decode: one wavefront per record; out[i] = sum_j y_j S[i][j] with St[j][i] = S[i][j] ---- */
__global__ __launch_bounds__(64) void pq_general_decode_kernel(GenFormat f, const uint8_t *rec, int64_t n, const float *St,
                                                               int rotated, float *out)
{
    __shared__ float buf[2][PQ_D];
    const int64_t v = blockIdx.x;
    const int tid = threadIdx.x;
    if (v >= n) return;
    const int cur = gen_dequant_rotated(f, rec + v * f.rec_bytes, buf, tid);
    float a0 = 0.f, a1 = 0.f;
    if (rotated) {
        a0 = buf[cur][2 * tid];
        a1 = buf[cur][2 * tid + 1];
    } else {
        for (int j = 0; j < PQ_D; ++j) {
            const float2 s2 = *reinterpret_cast<const float2 *>(St + j * PQ_D + 2 * tid);
            a0 = fmaf(buf[cur][j], s2.x, a0);
            a1 = fmaf(buf[cur][j], s2.y, a1);
        }
    }
    out[v * PQ_D + 2 * tid] = a0;
    out[v * PQ_D + 2 * tid + 1] = a1;
}

__device__ __forceinline__ float gen_wave_sum(float x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
    return x;
}

/* ---- attention: one workgroup of kGenAttnWaves wavefronts per (sequence, query head).  Wavefront w takes tokens
   w, w + kGenAttnWaves, ... one after another (DeQuant of the key, score, DeQuant of the value, running softmax);
   the wavefronts' partial results are then merged in wavefront order, so the result does not depend on timing. ---- */
constexpr int kGenAttnWaves = 16;

__global__ __launch_bounds__(kGenAttnWaves * 64) void pq_general_attn_kernel(GenFormat f, const uint16_t *q, float *out,
                                                                             const uint8_t *k_rec, const uint8_t *v_rec,
                                                                             const int64_t *seq_start, const int32_t *ctx_len,
                                                                             int Hq, int Hkv, int64_t pool_tokens, float scale,
                                                                             const float *S, const float *St)
{
    __shared__ float sq[PQ_D];
    __shared__ float sqr[PQ_D];                         /* q' = q S */
    __shared__ float buf[kGenAttnWaves][2][PQ_D];       /* a wavefront's DeQuant buffers */
    __shared__ float part_o[kGenAttnWaves][PQ_D];
    __shared__ float part_ml[kGenAttnWaves][2];
    const int row = blockIdx.x, b = row / Hq, head = row % Hq, hk = head / (Hq / Hkv);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < PQ_D) sq[tid] = __uint_as_float((uint32_t)q[(int64_t)row * PQ_D + tid] << 16);
    __syncthreads();
    if (tid < 64) {
        float a0 = 0.f, a1 = 0.f; /* this thread's two coordinates of q' */
        for (int i = 0; i < PQ_D; ++i) {
            const float2 s2 = *reinterpret_cast<const float2 *>(S + i * PQ_D + 2 * tid);
            a0 = fmaf(sq[i], s2.x, a0);
            a1 = fmaf(sq[i], s2.y, a1);
        }
        sqr[2 * tid] = a0;
        sqr[2 * tid + 1] = a1;
    }
    __syncthreads();
    const float q0 = sqr[2 * lane], q1 = sqr[2 * lane + 1];
    int64_t n = ctx_len[b];
    const int64_t t0 = seq_start[b];
    if (n < 0 || t0 < 0 || t0 + n > pool_tokens) n = 0; /* a sequence outside the pool is treated as empty */
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int64_t t = wave; t < n; t += kGenAttnWaves) {
        const int64_t slot = (int64_t)hk * pool_tokens + t0 + t;
        int cur = gen_dequant_rotated(f, k_rec + slot * f.rec_bytes, buf[wave], lane);
        const float s = gen_wave_sum(q0 * buf[wave][cur][2 * lane] + q1 * buf[wave][cur][2 * lane + 1]) * scale;
        gen_wave_sync();
        cur = gen_dequant_rotated(f, v_rec + slot * f.rec_bytes, buf[wave], lane);
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new), p = expf(s - m_new); /* exp(-inf) = 0 at the first token */
        l = l * alpha + p;
        o0 = o0 * alpha + p * buf[wave][cur][2 * lane];
        o1 = o1 * alpha + p * buf[wave][cur][2 * lane + 1];
        m = m_new;
        gen_wave_sync();
    }
    part_o[wave][2 * lane] = o0;
    part_o[wave][2 * lane + 1] = o1;
    if (lane == 0) { part_ml[wave][0] = m; part_ml[wave][1] = l; }
    __syncthreads();
    if (tid < 64) {
        float mm = -INFINITY;
        for (int w = 0; w < kGenAttnWaves; ++w) mm = fmaxf(mm, part_ml[w][0]);
        float lt = 0.f, a0 = 0.f, a1 = 0.f;
        for (int w = 0; w < kGenAttnWaves; ++w) {
            const float mw = part_ml[w][0];
            const float wgt = mw == -INFINITY ? 0.f : expf(mw - mm); /* a wavefront without a token */
            lt = fmaf(part_ml[w][1], wgt, lt);
            a0 = fmaf(part_o[w][2 * tid], wgt, a0);
            a1 = fmaf(part_o[w][2 * tid + 1], wgt, a1);
        }
        sq[2 * tid] = lt > 0.f ? a0 / lt : 0.f;   /* o' in the rotated domain (sq is free by now) */
        sq[2 * tid + 1] = lt > 0.f ? a1 / lt : 0.f;
    }
    __syncthreads();
    if (tid < 64) {
        float a0 = 0.f, a1 = 0.f;
        for (int j = 0; j < PQ_D; ++j) {
            const float2 s2 = *reinterpret_cast<const float2 *>(St + j * PQ_D + 2 * tid);
            a0 = fmaf(sq[j], s2.x, a0);
            a1 = fmaf(sq[j], s2.y, a1);
        }
        out[(int64_t)row * PQ_D + 2 * tid] = a0;
        out[(int64_t)row * PQ_D + 2 * tid + 1] = a1;
    }
}

} // namespace

extern "C" size_t pq_general_record_bytes(const pq_general_format *f)
{
    if (!general_format_ok(f)) return 0;
    return (size_t)((general_code_bits(f) + 7) / 8 + 2 * (PQ_D >> f->depth));
}

extern "C" int pq_general_codebook_entries(const pq_general_format *f)
{
    if (!general_format_ok(f)) return 0;
    int n = 0;
    for (int l = 0; l < f->depth; ++l) n += 1 << f->bits[l];
    return n;
}

extern "C" pq_status pq_general_codebooks(const pq_general_format *f, double *cbg)
{
    if (!general_format_ok(f) || !cbg) return PQ_EINVAL;
    const double two_pi = 6.28318530717958647692;
    int off = 0;
    for (int l = 0; l < f->depth; ++l) {
        const int K = 1 << f->bits[l];
        if (l == 0) {
            for (int k = 0; k < K; ++k) cbg[off + k] = two_pi * (k + 0.5) / K; /* uniform on [0, 2 pi): equal cells */
        } else {
            double bnd[kGenMaxCells + 1];
            pq_lloyd_max(l + 1, K, cbg + off, bnd);
        }
        off += K;
    }
    return PQ_OK;
}

extern "C" pq_status pq_general_encode(const pq_ctx *ctx, const pq_general_format *f, const double *cbg, const void *x,
                                       pq_dtype xt, int64_t n_vectors, int64_t ld_vector, uint8_t *records,
                                       void *hip_stream)
{
    if (!ctx || !x || !records || n_vectors < 0 || ld_vector < PQ_D) return PQ_EINVAL;
    if (xt != PQ_F32 && xt != PQ_BF16) return PQ_EINVAL;
    if (n_vectors > 0x7FFFFFFF) return PQ_EUNSUPPORTED;
    GenFormat g;
    pq_status st = make_format(f, cbg, &g);
    if (st != PQ_OK) return st;
    if (n_vectors == 0) return PQ_OK;
    const PqDeviceState *ds = nullptr;
    st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (xt == PQ_BF16)
        hipLaunchKernelGGL(pq_general_encode_kernel<PQ_BF16>, dim3((unsigned)n_vectors), dim3(64), 0, s, g, x, ld_vector, n_vectors, ds->S_f32, records);
    else
        hipLaunchKernelGGL(pq_general_encode_kernel<PQ_F32>, dim3((unsigned)n_vectors), dim3(64), 0, s, g, x, ld_vector, n_vectors, ds->S_f32, records);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

extern "C" pq_status pq_general_decode(const pq_ctx *ctx, const pq_general_format *f, const double *cbg,
                                       const uint8_t *records, int64_t n_vectors, int rotated, float *out, void *hip_stream)
{
    if (!ctx || !records || !out || n_vectors < 0) return PQ_EINVAL;
    if (n_vectors > 0x7FFFFFFF) return PQ_EUNSUPPORTED;
    GenFormat g;
    pq_status st = make_format(f, cbg, &g);
    if (st != PQ_OK) return st;
    if (n_vectors == 0) return PQ_OK;
    const PqDeviceState *ds = nullptr;
    st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    hipLaunchKernelGGL(pq_general_decode_kernel, dim3((unsigned)n_vectors), dim3(64), 0, static_cast<hipStream_t>(hip_stream),
                       g, records, n_vectors, ds->St_f32, rotated, out);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

extern "C" pq_status pq_general_attn_decode(const pq_ctx *ctx, const pq_general_format *f, const double *cbg, const void *q,
                                            float *out, const uint8_t *k_records, const uint8_t *v_records,
                                            const int64_t *seq_start, const int32_t *ctx_len, int B, int Hq, int Hkv,
                                            int64_t pool_tokens, float softmax_scale, void *hip_stream)
{
    if (!ctx || !q || !out || !k_records || !v_records || !seq_start || !ctx_len) return PQ_EINVAL;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || pool_tokens <= 0) return PQ_EINVAL;
    if ((int64_t)B * Hq > 0x7FFFFFFF) return PQ_EUNSUPPORTED;
    GenFormat g;
    pq_status st = make_format(f, cbg, &g);
    if (st != PQ_OK) return st;
    const PqDeviceState *ds = nullptr;
    st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    hipLaunchKernelGGL(pq_general_attn_kernel, dim3((unsigned)(B * Hq)), dim3(kGenAttnWaves * 64), 0, static_cast<hipStream_t>(hip_stream), g,
                       static_cast<const uint16_t *>(q), out, k_records, v_records, seq_start, ctx_len, Hq, Hkv, pool_tokens,
                       softmax_scale, ds->S_f32, ds->St_f32);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}
