/*
 * pq_fit.hip -- pq_fit_codebooks: online codebook construction (Section 4.1,
 * line 3 of Algorithm 1 in its online variant: 1-D k-means on the angles of the
 * polar-transformed inputs), for gfx950.
 *
 * The heavy part runs on the GPU: every input vector is rotated (y = x S), its
 * 120 angles are formed (procedure Polar) and counted into fine histograms,
 * one per level (8192 bins over [0, 2 pi) for level 1, 2048 over [0, pi/2] for
 * levels 2-4; for a full-depth context 2048 more for each of levels 5-7, see
 * pq_fit_codebooks_deep).  The k-means rounds then run on the bin counts on the host
 * in fp64, which costs well under a millisecond and is where the result is
 * wanted (pq_set_codebooks takes host centroids).
 *
 * Kernel: one wavefront per tile of 64 vectors, sixteen wavefronts per
 * workgroup, S and the histograms in LDS.
 *   Rotation on the matrix cores as in the encode kernel (same operand image of
 *   S, same register layout of the result: a lane ends up with complete blocks
 *   of 16 rotated coordinates of one vector), with the two leading bf16 terms
 *   of S (16 significant bits; bf16 inputs are exact operands, fp32 inputs are
 *   split into two terms and the three products above 2^-16 are used): the
 *   angle error of 1e-5 rad is a hundredth of a bin.
 *   Bins are uniform in the pseudo-angle t = v / (u + v) of a node's two inputs
 *   (level 1: quadrant + t, with |y| or |x| on top so that it grows with the
 *   angle), which is monotone in the angle and costs a reciprocal instead of
 *   an arctangent: bin edge k / 2048 is the angle atan2(k, 2048 - k).  The
 *   host part knows the edges and treats the angles of a bin as spread evenly
 *   between them.
 * Counts are integers: the result does not depend on scheduling.
 */
#include "pq_common.h"

#include <cmath>
#include <cstring>
#include <vector>

namespace {

constexpr int kBins1 = 8192, kBinsU = 2048;
constexpr int kHistSize = kBins1 + 3 * kBinsU; /* 14336 counters */
constexpr int kHistUpper = 3 * kBinsU;         /* levels 5..7 (full-depth recursion): 6144 more */
constexpr int kFitWaves = 16, kFitThreads = kFitWaves * 64;
constexpr int kTileVecs = 64;
constexpr int kFitTerms = 2;                   /* bf16 terms of S that take part */

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct FitArgs {
    const void *x;
    int64_t ld_token, ld_head, n_tokens;
    int n_heads;
    int64_t tiles_per_head, n_items;
    const uint4 *S_bf16x3; /* the encode kernel's operand image of S, term-major */
    uint32_t *hist;        /* [kHistSize], zeroed before the launch */
    uint32_t *hist_up;     /* [kHistUpper] or NULL: angles of levels 5..7 */
};

union FitOperand {
    bf16x8 v;
    uint4 q;
    uint32_t w[4];
};

__device__ __forceinline__ uint32_t fit_bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

/* bin of the angle of (u, v), both >= 0, among kBinsU bins uniform in t = v / (u + v); atan2(0, 0) counts as 0 */
__device__ __forceinline__ int upper_bin(float u, float v)
{
    const float t = v * __builtin_amdgcn_rcpf(fmaxf(u + v, 1e-37f));
    return min((int)(t * (float)kBinsU), kBinsU - 1);
}

/* Angles of one block of 16 rotated coordinates into the LDS histograms; returns the block's radius. */
__device__ __forceinline__ float count_block_angles(const f32x16 &y, uint32_t *sh)
{
    float r[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const float a = y[2 * p], b = y[2 * p + 1];
        const float fa = fabsf(a), fb = fabsf(b);
        const uint32_t sa = __float_as_uint(a) >> 31, sb = __float_as_uint(b) >> 31;
        const uint32_t odd = sa ^ sb, quadrant = 2u * sb + odd; /* [0, 2 pi): (+,+), (-,+), (-,-), (+,-) */
        const float t = (odd ? fa : fb) * __builtin_amdgcn_rcpf(fmaxf(fa + fb, 1e-37f));
        const int bin = (int)quadrant * (kBins1 / 4) + min((int)(t * (float)(kBins1 / 4)), kBins1 / 4 - 1);
        atomicAdd(&sh[bin], 1u);
        r[p] = sqrtf(a * a + b * b);
    }
    int base = kBins1;
#pragma unroll
    for (int n = 4; n >= 1; n >>= 1) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (p < n) {
                const float u = r[2 * p], v = r[2 * p + 1];
                atomicAdd(&sh[base + upper_bin(u, v)], 1u);
                r[p] = sqrtf(u * u + v * v);
            }
        }
        base += kBinsU;
    }
    return r[0];
}

template <int XT>
__global__ __launch_bounds__(kFitThreads, 1) void pq_angle_histogram_kernel(FitArgs a)
{
    __shared__ uint4 sS[kFitTerms * 4 * 8 * 64];    /* 64 KB */
    __shared__ uint32_t sh[kHistSize + kHistUpper]; /* 80 KB */
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    {
        uint4 stage[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) stage[i] = a.S_bf16x3[tid + i * kFitThreads];
#pragma unroll
        for (int i = 0; i < 4; ++i) sS[tid + i * kFitThreads] = stage[i];
    }
    for (int c = tid; c < kHistSize + kHistUpper; c += kFitThreads) sh[c] = 0u;
    __syncthreads();

    const int j = lane & 31, H = lane >> 5; /* vector within a 32-vector half, lane half */
    constexpr int NXT = (XT == PQ_BF16) ? 1 : 2; /* bf16 terms of x */
    for (int64_t item = (int64_t)blockIdx.x * kFitWaves + wave; item < a.n_items; item += (int64_t)gridDim.x * kFitWaves) {
        const int head = (int)(item / a.tiles_per_head);
        const int64_t t0 = (item % a.tiles_per_head) * kTileVecs;
        float rb[2][4]; /* radii of blocks 4H .. 4H+3 of this lane's two vectors */
        bool valid[2];
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int64_t tok = t0 + 32 * v + j;
            valid[v] = tok < a.n_tokens;
            /* a lane without a vector reads the tile's first one again and counts nothing */
            const int64_t at = (valid[v] ? tok : t0) * a.ld_token + (int64_t)head * a.ld_head;
            /* B operands: this lane's 8-coordinate slices (coordinates 64 H + 8 ks .. + 7) of its vector */
            FitOperand xb[NXT][8];
            if constexpr (XT == PQ_BF16) {
                const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.x) + at);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) xb[0][ks].q = xr[8 * H + ks];
            } else {
                const float4 *xr = reinterpret_cast<const float4 *>(static_cast<const float *>(a.x) + at);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const float4 p0 = xr[16 * H + 2 * ks], p1 = xr[16 * H + 2 * ks + 1];
                    const float f[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        uint32_t hi[2], lo[2];
#pragma unroll
                        for (int z = 0; z < 2; ++z) {
                            hi[z] = fit_bf16_rne(f[e + z]);
                            lo[z] = fit_bf16_rne(f[e + z] - __uint_as_float(hi[z] << 16));
                        }
                        xb[0][ks].w[e / 2] = hi[0] | (hi[1] << 16);
                        xb[NXT - 1][ks].w[e / 2] = lo[0] | (lo[1] << 16);
                    }
                }
            }
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
                /* D[i][j] = sum_k S[k][col(rt, i)] x[j][k]: lane (H, j) receives rotated coordinates
                   16 (4 H + rt) .. + 15 of vector j */
                f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                    for (int term = kFitTerms - 1; term >= 0; --term)
#pragma unroll
                        for (int xt = 0; xt < NXT; ++xt) {
                            if (term + xt > 1) continue; /* below 2^-16 of the leading product */
                            FitOperand sa;
                            sa.q = sS[((term * 4 + rt) * 8 + ks) * 64 + lane];
                            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa.v, xb[xt][ks].v, acc, 0, 0, 0);
                        }
                const float r = valid[v] ? count_block_angles(acc, sh) : 0.f;
                rb[v][rt] = r;
            }
        }
        if (a.hist_up) {
            /* levels 5 and 6 inside the lane (blocks 4H .. 4H+3), level 7 joins the two lane halves */
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const float r50 = sqrtf(rb[v][0] * rb[v][0] + rb[v][1] * rb[v][1]);
                const float r51 = sqrtf(rb[v][2] * rb[v][2] + rb[v][3] * rb[v][3]);
                const float r6 = sqrtf(r50 * r50 + r51 * r51);
                const float other = __shfl_xor(r6, 32);
                if (valid[v]) {
                    uint32_t *up = sh + kHistSize;
                    atomicAdd(&up[upper_bin(rb[v][0], rb[v][1])], 1u);
                    atomicAdd(&up[upper_bin(rb[v][2], rb[v][3])], 1u);
                    atomicAdd(&up[kBinsU + upper_bin(r50, r51)], 1u);
                    if (H == 0) atomicAdd(&up[2 * kBinsU + upper_bin(r6, other)], 1u);
                }
            }
        }
    }
    __syncthreads();
    for (int c = tid; c < kHistSize; c += kFitThreads)
        if (sh[c]) atomicAdd(&a.hist[c], sh[c]);
    if (a.hist_up)
        for (int c = tid; c < kHistUpper; c += kFitThreads)
            if (sh[kHistSize + c]) atomicAdd(&a.hist_up[c], sh[kHistSize + c]);
}

/* angle of the lower edge of bin b of a level's histogram (b = bins gives the upper end of the range) */
double bin_edge(int b, int bins, bool level1)
{
    const double half_pi = 1.57079632679489661923132169163975144;
    const int per = level1 ? bins / 4 : bins; /* bins per quarter turn */
    const int q = b / per, k = b % per;
    return q * half_pi + atan2((double)k, (double)(per - k));
}

/* k-means rounds on one level's histogram.  The angles of a bin are taken as spread evenly over
   it: a bin that a cell boundary (midpoint of two centroids) cuts gives each side its share of
   the count, centred on its part of the bin; an uncut bin stands for its centre.  Nearest
   centroid by linear distance (procedure Quant); a centroid whose cell is empty stays. */
void lloyd_on_histogram(const uint32_t *hist, int bins, bool level1, int K, int iterations, double *c)
{
    std::vector<double> edges((size_t)bins + 1);
    for (int b = 0; b <= bins; ++b) edges[b] = bin_edge(b, bins, level1);
    for (int it = 0; it < iterations; ++it) {
        double sum[16] = {0};
        double num[16] = {0};
        double edge[17];
        edge[0] = -1.0;
        edge[K] = 1e300;
        for (int k = 1; k < K; ++k) edge[k] = 0.5 * (c[k - 1] + c[k]);
        int k = 0;
        for (int b = 0; b < bins; ++b) {
            if (!hist[b]) continue;
            const double lo = edges[b], hi = edges[b + 1], per_rad = (double)hist[b] / (hi - lo);
            while (k + 1 < K && edge[k + 1] <= lo) ++k;
            double from = lo;
            int q = k;
            while (from < hi) { /* the parts of [lo, hi) that fall into cells q, q+1, ... */
                const double to = edge[q + 1] < hi ? edge[q + 1] : hi;
                const double mass = per_rad * (to - from);
                sum[q] += mass * 0.5 * (from + to);
                num[q] += mass;
                from = to;
                if (from < hi) ++q;
            }
        }
        for (int q = 0; q < K; ++q)
            if (num[q] > 0) c[q] = sum[q] / num[q];
    }
}

} // namespace

extern "C" size_t pq_fit_workspace_bytes(void) { return (size_t)(kHistSize + kHistUpper) * sizeof(uint32_t); }

namespace {

/* clears the histograms with a kernel of the library's own: a memset node would not survive graph capture */
__global__ __launch_bounds__(256) void pq_fit_clear_kernel(uint32_t *hist, int n)
{
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) hist[i] = 0u;
}

pq_status check_start(const pq_ctx *ctx, const double *cb_init, const double *cbt_init, bool upper, double (&c)[28],
                      double (&ct)[3][8])
{
    if (cb_init) {
        memcpy(c, cb_init, sizeof(c));
    } else {
        for (int k = 0; k < 16; ++k) c[k] = ctx->centroids[0][k];
        for (int l = 1; l < 4; ++l)
            for (int k = 0; k < 4; ++k) c[16 + 4 * (l - 1) + k] = ctx->centroids[l][k];
    }
    const int off[4] = {0, 16, 20, 24}, K[4] = {16, 4, 4, 4};
    for (int l = 0; l < 4; ++l)
        for (int k = 0; k < K[l]; ++k) {
            if (!std::isfinite(c[off[l] + k])) return PQ_EINVAL;
            if (k > 0 && !(c[off[l] + k] > c[off[l] + k - 1])) return PQ_EINVAL;
        }
    if (upper) {
        for (int l = 0; l < 3; ++l) {
            const int Kl = 1 << ctx->upper_bits[l];
            for (int k = 0; k < 8; ++k) ct[l][k] = cbt_init ? cbt_init[8 * l + k] : (k < Kl ? ctx->upper_centroids[l][k] : 0.0);
            for (int k = 0; k < Kl; ++k) {
                if (!std::isfinite(ct[l][k])) return PQ_EINVAL;
                if (k > 0 && !(ct[l][k] > ct[l][k - 1])) return PQ_EINVAL;
            }
        }
    }
    return PQ_OK;
}

} // namespace

extern "C" pq_status pq_fit_count_angles(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                                         int64_t ld_token, int64_t ld_head, void *workspace, size_t workspace_bytes,
                                         void *hip_stream)
{
    if (!ctx || !x || !workspace) return PQ_EINVAL;
    if (xt != PQ_F32 && xt != PQ_BF16) return PQ_EINVAL;
    if (n_tokens <= 0 || n_heads <= 0 || ld_token < 0 || ld_head < 0) return PQ_EINVAL;
    if (workspace_bytes < pq_fit_workspace_bytes()) return PQ_ENOMEM;
    const int64_t elems16 = xt == PQ_BF16 ? 8 : 4;
    if (!pq_aligned16(workspace) || !pq_aligned16(x) || (ld_token % elems16) || (ld_head % elems16)) return PQ_EALIGN;
    /* every bin counter must hold the angles of a level: 64 per vector at level 1 */
    if ((double)n_tokens * n_heads * 64.0 >= 4294967295.0) return PQ_EUNSUPPORTED;
    const bool upper = ctx->depth == 7;
    const PqDeviceState *ds = nullptr;
    pq_status st = pq_device_state(ctx, &ds);
    if (st != PQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    uint32_t *hist = static_cast<uint32_t *>(workspace);
    hipLaunchKernelGGL(pq_fit_clear_kernel, dim3(16), dim3(256), 0, s, hist, kHistSize + kHistUpper);
    FitArgs a{};
    a.x = x; a.ld_token = ld_token; a.ld_head = ld_head; a.n_tokens = n_tokens; a.n_heads = n_heads;
    a.tiles_per_head = (n_tokens + kTileVecs - 1) / kTileVecs;
    a.n_items = a.tiles_per_head * n_heads;
    a.S_bf16x3 = reinterpret_cast<const uint4 *>(ds->S_bf16x3);
    a.hist = hist;
    a.hist_up = upper ? hist + kHistSize : nullptr;
    int64_t blocks = (a.n_items + kFitWaves - 1) / kFitWaves;
    if (blocks > 256) blocks = 256;
    if (xt == PQ_BF16) hipLaunchKernelGGL(pq_angle_histogram_kernel<PQ_BF16>, dim3((unsigned)blocks), dim3(kFitThreads), 0, s, a);
    else hipLaunchKernelGGL(pq_angle_histogram_kernel<PQ_F32>, dim3((unsigned)blocks), dim3(kFitThreads), 0, s, a);
    PQ_HIP_TRY(hipGetLastError());
    return PQ_OK;
}

extern "C" pq_status pq_fit_cluster(const pq_ctx *ctx, const uint32_t *hist, const double *cb_init, const double *cbt_init,
                                    int iterations, double *cb_out, double *cbt_out)
{
    if (!ctx || !hist || !cb_out || iterations < 0) return PQ_EINVAL;
    const bool upper = ctx->depth == 7;
    if (upper && !cbt_out) return PQ_EINVAL;
    double c[28], ct[3][8] = {};
    const pq_status st = check_start(ctx, cb_init, cbt_init, upper, c, ct);
    if (st != PQ_OK) return st;
    const int off[4] = {0, 16, 20, 24};
    lloyd_on_histogram(hist, kBins1, true, 16, iterations, c);
    for (int l = 1; l < 4; ++l)
        lloyd_on_histogram(hist + kBins1 + (l - 1) * kBinsU, kBinsU, false, 4, iterations, c + off[l]);
    memcpy(cb_out, c, sizeof(c));
    if (upper) {
        for (int l = 0; l < 3; ++l)
            lloyd_on_histogram(hist + kHistSize + l * kBinsU, kBinsU, false, 1 << ctx->upper_bits[l], iterations, ct[l]);
        memcpy(cbt_out, ct, sizeof(ct));
    }
    return PQ_OK;
}

namespace {

/* the two steps with a copy of the histograms and a wait for the stream in between */
pq_status fit_codebooks(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                        int64_t ld_token, int64_t ld_head, const double *cb_init, const double *cbt_init, bool upper,
                        int iterations, double *cb_out, double *cbt_out, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    if (!ctx || !cb_out || (upper && !cbt_out) || iterations < 0) return PQ_EINVAL;
    if (upper && ctx->depth != 7) return PQ_EINVAL;
    double unused_upper[3][8];
    if (!upper && ctx->depth == 7) cbt_out = &unused_upper[0][0]; /* levels 1..4 only were asked for */
    double c[28], ct[3][8] = {};
    pq_status st = check_start(ctx, cb_init, cbt_init, upper, c, ct); /* before anything is launched */
    if (st != PQ_OK) return st;
    st = pq_fit_count_angles(ctx, x, xt, n_tokens, n_heads, ld_token, ld_head, workspace, workspace_bytes, hip_stream);
    if (st != PQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    std::vector<uint32_t> h(kHistSize + kHistUpper);
    PQ_HIP_TRY(hipMemcpyAsync(h.data(), workspace, pq_fit_workspace_bytes(), hipMemcpyDeviceToHost, s));
    PQ_HIP_TRY(hipStreamSynchronize(s));
    return pq_fit_cluster(ctx, h.data(), cb_init, cbt_init, iterations, cb_out, cbt_out);
}

} // namespace

extern "C" pq_status pq_fit_codebooks(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                                      int64_t ld_token, int64_t ld_head, const double *cb_init, int iterations,
                                      double *cb_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return fit_codebooks(ctx, x, xt, n_tokens, n_heads, ld_token, ld_head, cb_init, nullptr, false, iterations, cb_out,
                         nullptr, workspace, workspace_bytes, hip_stream);
}

extern "C" pq_status pq_fit_codebooks_deep(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                                           int64_t ld_token, int64_t ld_head, const double *cb_init,
                                           const double *cbt_init, int iterations, double *cb_out, double *cbt_out,
                                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return fit_codebooks(ctx, x, xt, n_tokens, n_heads, ld_token, ld_head, cb_init, cbt_init, true, iterations, cb_out,
                         cbt_out, workspace, workspace_bytes, hip_stream);
}
