/*
 * pq_fit.hip -- pq_fit_codebooks: online codebook construction (Section 4.1,
 * line 3 of Algorithm 1 in its online variant: 1-D k-means on the angles of the
 * polar-transformed inputs), for gfx950.
 *
 * The heavy part runs on the GPU: every input vector is rotated (y = x S, fp32),
 * its 120 angles are formed (procedure Polar) and counted into fine histograms,
 * one per level (8192 bins over [0, 2 pi) for level 1, 2048 over [0, pi/2] for
 * levels 2-4; for a full-depth context 2048 more for each of levels 5-7, see
 * pq_fit_codebooks_deep).  The k-means rounds then run on the bin counts on the host
 * in fp64 -- each bin stands for its centre -- which costs microseconds and is
 * where the result is wanted (pq_set_codebooks takes host centroids).
 *
 * Kernel: a workgroup keeps S (64 KB, fp32) and its four histograms (56 KB) in
 * LDS and walks over tiles of 32 vectors: the tile is staged as fp32, thread
 * (half, j) accumulates coordinate j of 16 vectors (S[i][j] from LDS once per
 * 16 products, x as LDS broadcasts), then thread (vector, block) runs the polar
 * recursion of one 16-coordinate block and bumps the bins with LDS atomics.
 * Counts are integers: the result does not depend on scheduling.
 */
#include "pq_common.h"

#include <cmath>
#include <cstring>
#include <vector>

namespace {

constexpr int kBins1 = 8192, kBinsU = 2048;
constexpr int kHistSize = kBins1 + 3 * kBinsU; /* 14336 counters */
constexpr int kHistUpper = 3 * kBinsU;         /* levels 5..7 (full-depth recursion): 6144 more, in global memory */
constexpr int kFitThreads = 256;
constexpr int kTileVecs = 32;
constexpr float kTwoPi = 6.28318530717958647692f, kHalfPi = 1.57079632679489661923f;

struct FitArgs {
    const void *x;
    int64_t ld_token, ld_head, n_tokens;
    int n_heads;
    int64_t tiles_per_head, n_items;
    const float *S;     /* S[i*128 + j] */
    uint32_t *hist;     /* [kHistSize], zeroed by the caller of the kernel */
    uint32_t *hist_up;  /* [kHistUpper] or NULL: angles of levels 5..7 */
};

template <int XT>
__global__ __launch_bounds__(kFitThreads) void pq_angle_histogram_kernel(FitArgs a)
{
    __shared__ float sS[PQ_D * PQ_D];
    __shared__ float sx[kTileVecs][PQ_D];
    __shared__ float sy[kTileVecs][PQ_D + 4]; /* +4: the 16-float rows of different vectors start in different banks */
    __shared__ uint32_t sh[kHistSize];
    const int tid = threadIdx.x;
    {   /* S: 16 float4 per thread, requested in two batches of 8 before they are stored */
        const float4 *src = reinterpret_cast<const float4 *>(a.S);
        float4 *dst = reinterpret_cast<float4 *>(sS);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float4 stage[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) stage[i] = src[tid + (8 * half + i) * kFitThreads];
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[tid + (8 * half + i) * kFitThreads] = stage[i];
        }
    }
    for (int c = tid; c < kHistSize; c += kFitThreads) sh[c] = 0u;
    __syncthreads();

    const int j = tid & 127, vhalf = tid >> 7;
    for (int64_t item = blockIdx.x; item < a.n_items; item += gridDim.x) {
        const int head = (int)(item / a.tiles_per_head);
        const int64_t t0 = (item % a.tiles_per_head) * kTileVecs;
        const int n_valid = (int)min((int64_t)kTileVecs, a.n_tokens - t0);
        /* stage the tile as fp32 (rows beyond the input are zero and are not counted below) */
        for (int c = tid; c < kTileVecs * PQ_D; c += kFitThreads) {
            const int v = c >> 7, k = c & 127;
            float val = 0.f;
            if (v < n_valid) {
                const int64_t at = (t0 + v) * a.ld_token + (int64_t)head * a.ld_head + k;
                if (XT == PQ_BF16) val = __uint_as_float((uint32_t)static_cast<const uint16_t *>(a.x)[at] << 16);
                else val = static_cast<const float *>(a.x)[at];
            }
            sx[v][k] = val;
        }
        __syncthreads();
        /* y[v][j] = sum_i x[v][i] S[i][j] for the 16 vectors of this thread's half */
        float acc[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        for (int i = 0; i < PQ_D; i += 4) {
            const float s0 = sS[(i + 0) * PQ_D + j], s1 = sS[(i + 1) * PQ_D + j];
            const float s2 = sS[(i + 2) * PQ_D + j], s3 = sS[(i + 3) * PQ_D + j];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float4 xv = *reinterpret_cast<const float4 *>(&sx[16 * vhalf + v][i]);
                acc[v] = fmaf(xv.x, s0, acc[v]);
                acc[v] = fmaf(xv.y, s1, acc[v]);
                acc[v] = fmaf(xv.z, s2, acc[v]);
                acc[v] = fmaf(xv.w, s3, acc[v]);
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) sy[16 * vhalf + v][j] = acc[v];
        __syncthreads();
        /* procedure Polar on block (tid & 7) of vector (tid >> 3); every angle goes into its bin */
        {
            const int v = tid >> 3, b = tid & 7;
            float rb = 0.f; /* radius of the block */
            if (v < n_valid) {
                float r[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) r[k] = sy[v][16 * b + k];
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    float ang = atan2f(r[2 * p + 1], r[2 * p]);
                    if (ang < 0.f) ang += kTwoPi;
                    int bin = (int)(ang * ((float)kBins1 / kTwoPi));
                    bin = bin < 0 ? 0 : (bin > kBins1 - 1 ? kBins1 - 1 : bin);
                    atomicAdd(&sh[bin], 1u);
                    r[p] = sqrtf(r[2 * p] * r[2 * p] + r[2 * p + 1] * r[2 * p + 1]);
                }
                int n = 4, base = kBins1;
#pragma unroll
                for (int l = 2; l <= 4; ++l) {
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        if (p < n) {
                            const float ang = atan2f(r[2 * p + 1], r[2 * p]); /* both >= 0: in [0, pi/2] */
                            int bin = (int)(ang * ((float)kBinsU / kHalfPi));
                            bin = bin < 0 ? 0 : (bin > kBinsU - 1 ? kBinsU - 1 : bin);
                            atomicAdd(&sh[base + bin], 1u);
                            r[p] = sqrtf(r[2 * p] * r[2 * p] + r[2 * p + 1] * r[2 * p + 1]);
                        }
                    }
                    n >>= 1;
                    base += kBinsU;
                }
                rb = r[0];
            }
            if (a.hist_up) {
                /* levels 5..7 join the eight block radii of a vector, which sit in eight neighbouring lanes:
                   the node of a level lives in the lane of its first block and fetches its sibling's radius
                   with a shuffle.  A vector gives 7 angles here: they are counted in global memory (the
                   LDS is full). */
                float r = rb;
#pragma unroll
                for (int l = 0; l < 3; ++l) {
                    const float sib = __shfl_xor(r, 1 << l);
                    if (v < n_valid && (b & ((2 << l) - 1)) == 0) {
                        const float ang = atan2f(sib, r); /* both >= 0: in [0, pi/2] */
                        int bin = (int)(ang * ((float)kBinsU / kHalfPi));
                        bin = bin < 0 ? 0 : (bin > kBinsU - 1 ? kBinsU - 1 : bin);
                        atomicAdd(&a.hist_up[l * kBinsU + bin], 1u);
                    }
                    r = sqrtf(r * r + sib * sib);
                }
            }
        }
        __syncthreads();
    }
    for (int c = tid; c < kHistSize; c += kFitThreads)
        if (sh[c]) atomicAdd(&a.hist[c], sh[c]);
}

/* k-means rounds on one level's histogram.  The angles of a bin are taken as spread evenly over
   it: a bin that a cell boundary (midpoint of two centroids) cuts gives each side its share of
   the count, centred on its part of the bin; an uncut bin stands for its centre.  Nearest
   centroid by linear distance (procedure Quant); a centroid whose cell is empty stays. */
void lloyd_on_histogram(const uint32_t *hist, int bins, double width, int K, int iterations, double *c)
{
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
            const double lo = b * width, hi = lo + width, per_rad = (double)hist[b] / width;
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
    a.S = ds->S_f32;
    a.hist = hist;
    a.hist_up = upper ? hist + kHistSize : nullptr;
    int64_t blocks = a.n_items < 256 ? a.n_items : 256;
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
    const double pi = 3.14159265358979323846264338327950288;
    lloyd_on_histogram(hist, kBins1, 2.0 * pi / kBins1, 16, iterations, c);
    for (int l = 1; l < 4; ++l)
        lloyd_on_histogram(hist + kBins1 + (l - 1) * kBinsU, kBinsU, 0.5 * pi / kBinsU, 4, iterations, c + off[l]);
    memcpy(cb_out, c, sizeof(c));
    if (upper) {
        for (int l = 0; l < 3; ++l)
            lloyd_on_histogram(hist + kHistSize + l * kBinsU, kBinsU, 0.5 * pi / kBinsU, 1 << ctx->upper_bits[l],
                               iterations, ct[l]);
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
